/*
 * CPU oracle for half-precision GEMM, C = A*B  (alpha = 1, beta = 0).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It shares no code, table or header with the
 * HIP path; only tests, the smoke check and the cpu_baseline leg of the
 * benchmark may build, load or call it.
 *
 * What it computes (paper Section 2.1, "HGEMM": C = alpha*A*B + beta*C with
 * alpha=1, beta=0; Section 2.3.2, Eq. 1: the reference is a CPU matmul of the
 * up-cast fp16 inputs):
 *
 *     C[i][j] = RNE_fp16( sum_{k=0}^{K-1} (double)A[i][k] * (double)B[k][j] )
 *
 * Each product of two fp16 numbers has at most 22 significant bits and is
 * exact in fp64; the sum runs left to right in fp64 and is rounded ONCE to
 * fp16 (round to nearest, ties to even; overflow to infinity; subnormals
 * kept; NaN in, NaN out).  The paper's Eq. 1 accumulates in fp32; fp64 is
 * used here because it is strictly closer to the exact sum, so that the
 * tolerance of a parity test measures the GPU's error and not the oracle's.
 *
 * fp16 <-> fp64 conversion is written out by hand on the bit patterns, so no
 * library half type is involved.  Everything is pinned by tests that do not
 * go through this file's arithmetic (exhaustive comparison with numpy's
 * float16, exact rational brute force, closed forms).
 *
 * Storage: A is M x K row-major with leading dimension lda (elements).
 * B is K x N row-major with leading dimension ldb, or, when b_col_major is
 * non-zero, stored N x K (element (k,j) at B[j*ldb + k]) -- the "TN" layout
 * of Section 2.2.2.  C is M x N row-major with leading dimension ldc.
 */
#include <stdint.h>
#include <string.h>

/* ---- fp16 bit pattern -> fp64 value ------------------------------------ */
double oracle_half_to_double(uint16_t h)
{
    const uint64_t sign = (uint64_t)(h >> 15) & 1u;
    const int      e    = (h >> 10) & 0x1f;   /* biased exponent, bias 15   */
    uint64_t       m    = h & 0x3ffu;         /* 10 explicit mantissa bits  */
    uint64_t       bits;

    if (e == 0x1f) {                          /* infinity or NaN            */
        bits = (sign << 63) | (0x7ffull << 52) | (m << 42);
    } else if (e != 0) {                      /* normal: 2^(e-15) * 1.m     */
        bits = (sign << 63) | ((uint64_t)(e - 15 + 1023) << 52) | (m << 42);
    } else if (m == 0) {                      /* signed zero                */
        bits = sign << 63;
    } else {                                  /* subnormal: m * 2^-24       */
        int shift = 0;                        /* normalise: find leading 1  */
        while ((m & 0x400u) == 0) { m <<= 1; ++shift; }
        m &= 0x3ffu;                          /* value = 1.m * 2^(-14-shift)*/
        bits = (sign << 63) | ((uint64_t)(-14 - shift + 1023) << 52) | (m << 42);
    }
    double d;
    memcpy(&d, &bits, sizeof d);
    return d;
}

/* ---- fp64 value -> nearest fp16 bit pattern (ties to even) --------------
 * One rounding step, straight from the 52-bit fp64 mantissa; never via fp32. */
uint16_t oracle_double_to_half(double x)
{
    uint64_t bits;
    memcpy(&bits, &x, sizeof bits);
    const uint16_t sign = (uint16_t)((bits >> 63) << 15);
    const int      e64  = (int)((bits >> 52) & 0x7ff);
    const uint64_t m64  = bits & 0xfffffffffffffull;

    if (e64 == 0x7ff) {                       /* inf / NaN                  */
        if (m64 == 0) return (uint16_t)(sign | 0x7c00u);
        uint16_t payload = (uint16_t)(m64 >> 42);
        return (uint16_t)(sign | 0x7c00u | 0x200u | payload); /* quiet NaN  */
    }
    if (e64 == 0) return sign;                /* fp64 zero/subnormal: < 2^-1022, far below half the smallest fp16 */

    int e = e64 - 1023;                       /* unbiased exponent          */
    if (e > 15) return (uint16_t)(sign | 0x7c00u);          /* >= 2^16      */
    if (e < -25) return sign;                 /* < 2^-25: below half of the smallest subnormal 2^-24 */

    /* 53-bit significand with the implicit one */
    uint64_t sig = m64 | (1ull << 52);
    /* number of low bits to discard so that the kept part is in units of
     * the target's last place: normal fp16 keeps 11 significant bits (drop
     * 42); below 2^-14 the last place is fixed at 2^-24, so drop more.     */
    int drop = 42;
    if (e < -14) drop += (-14 - e);           /* at most 42 + 11 = 53       */

    uint64_t kept = sig >> drop;
    uint64_t rem  = sig & ((1ull << drop) - 1);
    uint64_t half = 1ull << (drop - 1);
    if (rem > half || (rem == half && (kept & 1))) ++kept;

    uint16_t out;
    if (e < -14) {
        /* kept counts units of 2^-24; reaching 1024 lands exactly on the
         * smallest normal, whose bit pattern is 0x0400 = 1024.             */
        out = (uint16_t)kept;
    } else {
        /* kept is in [1024, 2048]; 2048 means the round carried up to the
         * next power of two.                                               */
        int be = e + 15;
        if (kept == 2048) { kept = 1024; ++be; }
        if (be >= 31) return (uint16_t)(sign | 0x7c00u);     /* overflow    */
        out = (uint16_t)((be << 10) | (kept & 0x3ffu));
    }
    return (uint16_t)(sign | out);
}

/* element (k,j) of B in either storage */
static inline uint16_t b_at(const uint16_t* B, int64_t ldb, int b_col_major,
                            int64_t k, int64_t j)
{
    return b_col_major ? B[j * ldb + k] : B[k * ldb + j];
}

/* One output element, the definition written out. */
static uint16_t dot_row_col(int64_t K, const uint16_t* A, int64_t lda,
                            const uint16_t* B, int64_t ldb, int b_col_major,
                            int64_t i, int64_t j)
{
    double s = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        s += oracle_half_to_double(A[i * lda + k]) *
             oracle_half_to_double(b_at(B, ldb, b_col_major, k, j));
    }
    return oracle_double_to_half(s);
}

/* Full product.  Rows are independent, so the optional OpenMP split over i
 * changes no element's arithmetic.  Returns 0, or -1 on bad arguments.     */
int oracle_hgemm(int64_t M, int64_t N, int64_t K,
                 const uint16_t* A, int64_t lda,
                 const uint16_t* B, int64_t ldb, int b_col_major,
                 uint16_t* C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (M == 0 || N == 0) return 0;
    if (!C || (K > 0 && (!A || !B))) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            C[i * ldc + j] = dot_row_col(K, A, lda, B, ldb, b_col_major, i, j);
        }
    }
    return 0;
}

/* The same definition at n chosen positions (ii[t], jj[t]); used where the
 * full product is too slow.  out[t] receives C[ii[t]][jj[t]].              */
int oracle_hgemm_at(int64_t M, int64_t N, int64_t K,
                    const uint16_t* A, int64_t lda,
                    const uint16_t* B, int64_t ldb, int b_col_major,
                    int64_t n, const int64_t* ii, const int64_t* jj,
                    uint16_t* out)
{
    if (M < 0 || N < 0 || K < 0 || n < 0) return -1;
    if (n == 0) return 0;
    if (!ii || !jj || !out || (K > 0 && (!A || !B))) return -1;
    for (int64_t t = 0; t < n; ++t)
        if (ii[t] < 0 || ii[t] >= M || jj[t] < 0 || jj[t] >= N) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        out[t] = dot_row_col(K, A, lda, B, ldb, b_col_major, ii[t], jj[t]);
    }
    return 0;
}

/* The unrounded fp64 sum at chosen positions: lets a test look at how close
 * a value sits to a rounding tie.                                          */
int oracle_hgemm_sum_at(int64_t M, int64_t N, int64_t K,
                        const uint16_t* A, int64_t lda,
                        const uint16_t* B, int64_t ldb, int b_col_major,
                        int64_t n, const int64_t* ii, const int64_t* jj,
                        double* out)
{
    if (M < 0 || N < 0 || K < 0 || n < 0) return -1;
    if (n == 0) return 0;
    if (!ii || !jj || !out || (K > 0 && (!A || !B))) return -1;
    for (int64_t t = 0; t < n; ++t)
        if (ii[t] < 0 || ii[t] >= M || jj[t] < 0 || jj[t] >= N) return -1;
    for (int64_t t = 0; t < n; ++t) {
        double s = 0.0;
        for (int64_t k = 0; k < K; ++k)
            s += oracle_half_to_double(A[ii[t] * lda + k]) *
                 oracle_half_to_double(b_at(B, ldb, b_col_major, k, jj[t]));
        out[t] = s;
    }
    return 0;
}

/* ---- the 16-bit accumulator variant --------------------------------------
 * Section 1 of the paper names fp16 and fp32 accumulators as both valid for
 * fp16 inputs, and its exact-match test (Section 2.3.2) keeps every output
 * at or below 2048 so that an fp16 accumulator can hold it exactly.  The
 * paper does not say how often such an accumulator is rounded; the reading
 * taken here: the running sum is an fp16 value that takes in `block`
 * products at a time,
 *
 *     acc <- RNE_fp16( (double)acc + sum_{k in block} (double)A[i][k]*(double)B[k][j] )
 *
 * with the block's products summed left to right in fp64 (exact products;
 * the fp64 sum of up to a few dozen of them is far below fp16 resolution).
 * block = 16 is the depth of one matrix-core instruction on the hardware this
 * repository targets; block = 1 rounds after every product; block >= K is
 * the fp64-accumulate definition above.  The last block may be short.      */
static uint16_t dot_row_col_acc16(int64_t K, int64_t block, const uint16_t* A, int64_t lda,
                                  const uint16_t* B, int64_t ldb, int b_col_major,
                                  int64_t i, int64_t j)
{
    uint16_t acc = 0;                                  /* +0.0 in fp16 */
    for (int64_t k0 = 0; k0 < K; k0 += block) {
        const int64_t k1 = (k0 + block < K) ? k0 + block : K;
        double s = 0.0;
        for (int64_t k = k0; k < k1; ++k) {
            s += oracle_half_to_double(A[i * lda + k]) *
                 oracle_half_to_double(b_at(B, ldb, b_col_major, k, j));
        }
        acc = oracle_double_to_half(oracle_half_to_double(acc) + s);
    }
    return acc;
}

int oracle_hgemm_acc16(int64_t M, int64_t N, int64_t K, int64_t block,
                       const uint16_t* A, int64_t lda,
                       const uint16_t* B, int64_t ldb, int b_col_major,
                       uint16_t* C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0 || block < 1) return -1;
    if (M == 0 || N == 0) return 0;
    if (!C || (K > 0 && (!A || !B))) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            C[i * ldc + j] = dot_row_col_acc16(K, block, A, lda, B, ldb, b_col_major, i, j);
        }
    }
    return 0;
}

int oracle_hgemm_acc16_at(int64_t M, int64_t N, int64_t K, int64_t block,
                          const uint16_t* A, int64_t lda,
                          const uint16_t* B, int64_t ldb, int b_col_major,
                          int64_t n, const int64_t* ii, const int64_t* jj,
                          uint16_t* out)
{
    if (M < 0 || N < 0 || K < 0 || n < 0 || block < 1) return -1;
    if (n == 0) return 0;
    if (!ii || !jj || !out || (K > 0 && (!A || !B))) return -1;
    for (int64_t t = 0; t < n; ++t)
        if (ii[t] < 0 || ii[t] >= M || jj[t] < 0 || jj[t] >= N) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        out[t] = dot_row_col_acc16(K, block, A, lda, B, ldb, b_col_major, ii[t], jj[t]);
    }
    return 0;
}

/* Bulk conversions, exported so the tests can pin them exhaustively.       */
void oracle_half_to_double_n(int64_t n, const uint16_t* h, double* d)
{
    for (int64_t t = 0; t < n; ++t) d[t] = oracle_half_to_double(h[t]);
}
void oracle_double_to_half_n(int64_t n, const double* d, uint16_t* h)
{
    for (int64_t t = 0; t < n; ++t) h[t] = oracle_double_to_half(d[t]);
}
