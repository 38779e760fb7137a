/*
 * NestedFP CPU oracle  --  TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT PATH.
 *
 * A plain, slow, scalar implementation of what the NestedFP hot path computes
 * (arxiv 2506.02024): the FP16 -> (upper, lower) byte-plane decomposition, its
 * lossless inverse, per-token E4M3 activation quantisation, and the linear-layer
 * GEMM in FP16 mode and in FP8 mode, accumulated in fp64.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or constant generator with the HIP library.
 *
 * Notation follows the paper: an FP16 word is S | E[4:0] | M[1:10] with M1 the
 * mantissa MSB (Sec. 2.1, Eq. 1); "upper" is the E4M3 byte S | E[3:0] | M'[1:3],
 * "lower" is M[3:10] (Sec. 4.1, "Our Proposal").
 *
 * Pins (see tests/test_oracle_*.py): every function here is checked against
 * something other than itself -- numpy's float16, PyTorch's CPU float8_e4m3fn
 * cast, the paper's lossless-reconstruction claim over all 65,536 FP16 words,
 * hand-derived words under tests/golden/, numpy float64 matmul, brute force.
 * The per-token activation-scale formula (amax/448) is the one reading the
 * paper does not fix: "parity unpinned" against the paper for that formula.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>

/* ------------------------------------------------------------------ */
/* Number formats (Sec. 2.1, Eq. 1)                                    */
/* ------------------------------------------------------------------ */

/* Value of an FP16 word by Eq. 1 with x=5, y=10, bias 15; E=0 is the IEEE
 * subnormal row (no hidden one, exponent 1-bias), E=31 is Inf/NaN. */
double oracle_fp16_value(uint16_t bits)
{
    int S = bits >> 15;
    int E = (bits >> 10) & 31;
    int Mant = bits & 1023;
    double frac = 0.0, v;
    for (int j = 1; j <= 10; ++j) {            /* sum_j M_j 2^-j */
        int Mj = (Mant >> (10 - j)) & 1;
        frac += Mj * ldexp(1.0, -j);
    }
    if (E == 31) v = (Mant == 0) ? INFINITY : NAN;
    else if (E == 0) v = frac * ldexp(1.0, 1 - 15);
    else v = (1.0 + frac) * ldexp(1.0, E - 15);
    return S ? -v : v;
}

/* Value of an E4M3 byte by Eq. 1 with x=4, y=3, bias 7 (the OCP "FN" flavour:
 * no infinities, S.1111.111 is NaN, largest finite magnitude 448).  The bias 7
 * is what makes the fixed 2^8 relation of Sec. 4.1 hold: 15 - 8 = 7. */
double oracle_e4m3_value(uint8_t code)
{
    int S = code >> 7;
    int E = (code >> 3) & 15;
    int Mant = code & 7;
    double frac = 0.0, v;
    for (int j = 1; j <= 3; ++j) {
        int Mj = (Mant >> (3 - j)) & 1;
        frac += Mj * ldexp(1.0, -j);
    }
    if (E == 15 && Mant == 7) v = NAN;
    else if (E == 0) v = frac * ldexp(1.0, 1 - 7);
    else v = (1.0 + frac) * ldexp(1.0, E - 7);
    return S ? -v : v;
}

/* Nearest E4M3 code to a finite real v, ties to the code with even mantissa
 * LSB, magnitudes beyond the largest finite value saturate to it (never the
 * NaN code).  Written as a search over the 127 finite magnitudes so that it
 * does not depend on any bit trick. */
uint8_t oracle_e4m3_encode(double v)
{
    static double mag[0x7F];                      /* the 127 finite magnitudes */
    static int have_mag = 0;                      /* filled on first use (callers are serial) */
    if (!have_mag) {
        for (int c = 0; c <= 0x7E; ++c) mag[c] = oracle_e4m3_value((uint8_t)c);
        have_mag = 1;
    }
    uint8_t sign = (v < 0.0 || (v == 0.0 && signbit(v))) ? 0x80 : 0x00;
    double a = fabs(v);
    int lo = 0;                                   /* largest code with value <= a */
    for (int c = 0; c <= 0x7E; ++c)
        if (mag[c] <= a) lo = c;
    if (lo == 0x7E) return sign | 0x7E;           /* saturate */
    double below = mag[lo];
    double above = mag[lo + 1];
    double d_lo = a - below, d_hi = above - a;
    int pick;
    if (d_lo < d_hi) pick = lo;
    else if (d_hi < d_lo) pick = lo + 1;
    else pick = (lo & 1) ? lo + 1 : lo;           /* tie: even code */
    return sign | (uint8_t)pick;
}

/* ------------------------------------------------------------------ */
/* The format (Sec. 4.1)                                               */
/* ------------------------------------------------------------------ */

/* Applicability (Sec. 4.1 "Opportunities", "Handling Exception Layers",
 * App. Table 4): a weight fits iff |w| <= 1.75.  Inf and NaN do not fit. */
int oracle_in_range(uint16_t bits)
{
    double v = oracle_fp16_value(bits);
    if (isnan(v) || isinf(v)) return 0;
    return fabs(v) <= 1.75;
}

/* Decomposition of one in-range FP16 word (Sec. 4.1 "Our Proposal"), field by
 * field: sign copied, the four low exponent bits copied (E's MSB is unused),
 * M[1:3] taken, then round-to-nearest-even on M[4:10] read as 0..127 against
 * the midpoint 64.  The rounding is applied to the constructed 7-bit value
 * E[3:0]|M[1:3], so a carry out of the mantissa moves into the exponent.
 * lower = the low 8 bits of the FP16 mantissa, M[3:10]. */
void oracle_decompose_one(uint16_t bits, uint8_t *upper, uint8_t *lower)
{
    int S = bits >> 15;
    int E = (bits >> 10) & 31;
    int Mant = bits & 1023;
    int E4 = E & 15;
    int M123 = Mant >> 7;
    int rest = Mant & 127;
    int constructed = (E4 << 3) | M123;
    int M3 = M123 & 1;
    int round_up;
    if (rest > 64) round_up = 1;
    else if (rest == 64) round_up = (M3 == 1);
    else round_up = 0;
    constructed = constructed + round_up;
    *upper = (uint8_t)((S << 7) | (constructed & 0x7F));
    *lower = (uint8_t)(Mant & 255);
}

/* Reconstruction of one FP16 word (Sec. 4.1 "FP16 Reconstruction"): the LSB of
 * upper is M3 after rounding, the MSB of lower is M3 before rounding; if they
 * differ the rounding went up and is undone by subtracting one from the 7-bit
 * E[3:0]|M[1:3] field.  Then S, a zero exponent MSB, E[3:0], M1, M2 and the
 * lower byte M[3:10] are put back in FP16 order. */
uint16_t oracle_reconstruct_one(uint8_t upper, uint8_t lower)
{
    int S = upper >> 7;
    int field = upper & 0x7F;
    int lsb_upper = field & 1;
    int msb_lower = lower >> 7;
    if (lsb_upper != msb_lower) field = (field - 1) & 0x7F;
    int E4 = field >> 3;
    int M12 = (field >> 1) & 3;
    return (uint16_t)((S << 15) | (0 << 14) | (E4 << 10) | (M12 << 8) | lower);
}

/* Whole-tensor forms.  W is [N,K] with row stride ldw (elements); planes are
 * dense [N,K].  Returns the number of out-of-range words (planes entries for
 * those are written as 0). */
uint64_t oracle_decompose(const uint16_t *W, int64_t N, int64_t K, int64_t ldw,
                          uint8_t *upper, uint8_t *lower)
{
    uint64_t bad = 0;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            uint16_t b = W[n * ldw + k];
            if (!oracle_in_range(b)) {
                ++bad;
                upper[n * K + k] = 0;
                lower[n * K + k] = 0;
            } else {
                oracle_decompose_one(b, &upper[n * K + k], &lower[n * K + k]);
            }
        }
    return bad;
}

uint64_t oracle_count_out_of_range(const uint16_t *W, int64_t N, int64_t K, int64_t ldw)
{
    uint64_t bad = 0;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            if (!oracle_in_range(W[n * ldw + k])) ++bad;
    return bad;
}

void oracle_reconstruct(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K,
                        uint16_t *W, int64_t ldw)
{
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            W[n * ldw + k] = oracle_reconstruct_one(upper[n * K + k], lower[n * K + k]);
}

/* ------------------------------------------------------------------ */
/* Activation quantisation for FP8 mode (Sec. 2.2 "E4M3 Format",        */
/* Sec. 5.1 "Methodology": per-token, dynamic)                          */
/* ------------------------------------------------------------------ */

/* Per row m of X: amax_m = max_k |X[m,k]|; scale_m = amax_m / 448 computed as
 * one IEEE binary32 division (scale_m = 1 when the row is all zero);
 * Xq[m,k] = E4M3(nearest-even, saturating)( binary32(X[m,k]) / scale_m ), the
 * quotient again one IEEE binary32 division.  If static_scale is non-NULL it
 * is used for every row instead (per-tensor static scaling).  X must be finite. */
void oracle_quantize_act(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                         const float *static_scale, uint8_t *Xq, float *scales)
{
    for (int64_t m = 0; m < M; ++m) {
        float s;
        if (static_scale) {
            s = *static_scale;
        } else {
            float amax = 0.0f;
            for (int64_t k = 0; k < K; ++k) {
                float a = (float)fabs(oracle_fp16_value(X[m * ldx + k]));
                if (a > amax) amax = a;
            }
            volatile float q = amax / 448.0f;       /* binary32 division */
            s = (amax == 0.0f) ? 1.0f : q;
        }
        scales[m] = s;
        for (int64_t k = 0; k < K; ++k) {
            float x = (float)oracle_fp16_value(X[m * ldx + k]);   /* exact */
            volatile float r = x / s;               /* binary32 division */
            Xq[m * K + k] = oracle_e4m3_encode((double)r);
        }
    }
}

/* ------------------------------------------------------------------ */
/* GEMM, both modes (Sec. 4 "Overview", Sec. 4.1 fixed scale 2^8)       */
/* ------------------------------------------------------------------ */

/* FP16 mode: because reconstruction is lossless, the result is the plain
 * product with the original FP16 weights:  Y[m,n] = sum_k X[m,k] * W[n,k],
 * here with every term and the running sum in fp64, k ascending. */
void oracle_gemm_fp16(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                      const uint16_t *W, int64_t N, int64_t ldw,
                      double *Y, int64_t ldy)
{
    /* every operand is decoded to fp64 once, then the textbook triple loop */
    double *Xd = (double *)malloc(sizeof(double) * (size_t)M * (size_t)K);
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            Xd[m * K + k] = oracle_fp16_value(X[m * ldx + k]);
#pragma omp parallel
    {
        double *w = (double *)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t k = 0; k < K; ++k)
                w[k] = oracle_fp16_value(W[n * ldw + k]);
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    acc += Xd[m * K + k] * w[k];
                Y[m * ldy + n] = acc;
            }
        }
        free(w);
    }
    free(Xd);
}

/* Same, but starting from the two planes (reconstruct, then multiply). */
void oracle_gemm_fp16_planes(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                             const uint8_t *upper, const uint8_t *lower, int64_t N,
                             double *Y, int64_t ldy)
{
    double *Xd = (double *)malloc(sizeof(double) * (size_t)M * (size_t)K);
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            Xd[m * K + k] = oracle_fp16_value(X[m * ldx + k]);
#pragma omp parallel
    {
        double *w = (double *)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t k = 0; k < K; ++k)
                w[k] = oracle_fp16_value(
                    oracle_reconstruct_one(upper[n * K + k], lower[n * K + k]));
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    acc += Xd[m * K + k] * w[k];
                Y[m * ldy + n] = acc;
            }
        }
        free(w);
    }
    free(Xd);
}

/* FP8 mode: the upper plane read as E4M3 is the weight times 2^8 (Sec. 4.1),
 * the activations are the quantised bytes with their row scales:
 *   Y[m,n] = scale_m * 2^-8 * sum_k e4m3(Xq[m,k]) * e4m3(upper[n,k]).
 * The lower plane is not an argument: FP8 mode never reads it. */
void oracle_gemm_fp8(const uint8_t *Xq, const float *scales, int64_t M, int64_t K,
                     const uint8_t *upper, int64_t N, double *Y, int64_t ldy)
{
    double *Xd = (double *)malloc(sizeof(double) * (size_t)M * (size_t)K);
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            Xd[m * K + k] = oracle_e4m3_value(Xq[m * K + k]);
#pragma omp parallel
    {
        double *w = (double *)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t k = 0; k < K; ++k)
                w[k] = oracle_e4m3_value(upper[n * K + k]);
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    acc += Xd[m * K + k] * w[k];
                Y[m * ldy + n] = (double)scales[m] * ldexp(1.0, -8) * acc;
            }
        }
        free(w);
    }
    free(Xd);
}

/* One sampled output element of each mode, for spot checks at full size. */
double oracle_dot_fp16(const uint16_t *x_row, const uint16_t *w_row, int64_t K)
{
    double acc = 0.0;
    for (int64_t k = 0; k < K; ++k)
        acc += oracle_fp16_value(x_row[k]) * oracle_fp16_value(w_row[k]);
    return acc;
}

double oracle_dot_fp8(const uint8_t *xq_row, float scale, const uint8_t *upper_row, int64_t K)
{
    double acc = 0.0;
    for (int64_t k = 0; k < K; ++k)
        acc += oracle_e4m3_value(xq_row[k]) * oracle_e4m3_value(upper_row[k]);
    return (double)scale * ldexp(1.0, -8) * acc;
}
