/*
 * CPU oracle for the ternary inner-product hot path of FATNN (arXiv 2008.05101).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are checked against.  It shares no code, header, table or helper
 * with the HIP library, and nothing on the product path may call it.
 *
 * The paper's fast inner product (Section 3.3, Eq. 3) is an identity: it reaches
 * exactly the ordinary integer dot product of two ternary vectors, only cheaper
 * (Remark 1).  So the oracle is that ordinary dot product, written out with
 * integer multiplies and no bit tricks:
 *
 *   weights      w = lw - 1   in {-1, 0, +1}           (lw = level index 0,1,2)
 *   activations  a = la - 1   in {-1, 0, +1}           symmetric mode
 *                a = la       in { 0, 1,  2}           ReLU mode (second
 *                                                      constraint, Section 3.3)
 *   C[m][n] = sum_k w[m][k] * a[n][k]
 *
 * The level index equals popcount(codec) of Table 1, so "level" and "codec" are
 * the same thing up to the free choice of 01 or 10 for the value 0.
 *
 * Convolution = im2col followed by that GEMM (Supplementary S1); here it is the
 * direct seven-loop definition with true zero padding (an out-of-bounds tap
 * contributes nothing).
 *
 * The conventional baseline of Eq. 2 with M = K = 2 is, as a result, again a
 * plain integer dot product, over the values that the 2-bit codes stand for.
 *
 * Pins (tests/test_oracle_*.py): Tables 1 and 2 of the paper, a literal
 * transcription of Eq. 3-7 and Algorithm 1 kept apart from this file, brute
 * force, closed forms, invariants and library integer matmul / convolution.
 * Every function here is pinned; the paper's speed numbers are not (other
 * hardware): "parity unpinned" applies to none of the functions below.
 */
#include <stddef.h>
#include <stdint.h>

enum { ORACLE_SYM = 0, ORACLE_RELU = 1 };
enum { ORACLE_BASIS_TERNARY = 0, ORACLE_BASIS_UNIFORM = 1 };

static inline int act_value(int level, int act_mode) {
    return act_mode == ORACLE_RELU ? level : level - 1;
}

/* Section 3.3, Eq. 3 (as the definition it equals).  Lw: [M][K], La: [N][K],
 * C: [M][N] row-major.  Returns 0, or -1 if a level is outside {0,1,2}. */
int oracle_ternary_gemm(const int8_t *Lw, const int8_t *La, int64_t M, int64_t N, int64_t K,
                        int act_mode, int32_t *C) {
    int bad = 0;
    for (int64_t i = 0; i < M * K; ++i)
        if (Lw[i] < 0 || Lw[i] > 2) bad = 1;
    for (int64_t i = 0; i < N * K; ++i)
        if (La[i] < 0 || La[i] > 2) bad = 1;
    if (bad) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k) {
                int w = (int)Lw[m * K + k] - 1;
                int a = act_value((int)La[n * K + k], act_mode);
                acc += (int64_t)(w * a);
            }
            C[m * N + n] = (int32_t)acc;
        }
    }
    return 0;
}

/* Supplementary S1: convolution as im2col + gemm, written as the direct
 * definition.  Lw: [Cout][R][S][Cin], Lx: [B][H][W][Cin], Y: [B][Ho][Wo][Cout].
 * Padding is the value 0 (the paper is silent; this is the convention its
 * im2col inherits). */
int oracle_ternary_conv2d(const int8_t *Lw, const int8_t *Lx, int64_t B, int64_t Cin, int64_t H,
                          int64_t W, int64_t Cout, int64_t R, int64_t S, int64_t stride,
                          int64_t pad, int act_mode, int32_t *Y) {
    int64_t Ho = (H + 2 * pad - R) / stride + 1;
    int64_t Wo = (W + 2 * pad - S) / stride + 1;
    int bad = 0;
    for (int64_t i = 0; i < Cout * R * S * Cin; ++i)
        if (Lw[i] < 0 || Lw[i] > 2) bad = 1;
    for (int64_t i = 0; i < B * H * W * Cin; ++i)
        if (Lx[i] < 0 || Lx[i] > 2) bad = 1;
    if (bad) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t ho = 0; ho < Ho; ++ho) {
            for (int64_t wo = 0; wo < Wo; ++wo) {
                for (int64_t o = 0; o < Cout; ++o) {
                    int64_t acc = 0;
                    for (int64_t r = 0; r < R; ++r) {
                        int64_t hi = ho * stride - pad + r;
                        if (hi < 0 || hi >= H) continue;
                        for (int64_t s = 0; s < S; ++s) {
                            int64_t wi = wo * stride - pad + s;
                            if (wi < 0 || wi >= W) continue;
                            const int8_t *wp = Lw + ((o * R + r) * S + s) * Cin;
                            const int8_t *xp = Lx + ((b * H + hi) * W + wi) * Cin;
                            for (int64_t c = 0; c < Cin; ++c) {
                                int w = (int)wp[c] - 1;
                                int a = act_value((int)xp[c], act_mode);
                                acc += (int64_t)(w * a);
                            }
                        }
                    }
                    Y[((b * Ho + ho) * Wo + wo) * Cout + o] = (int32_t)acc;
                }
            }
        }
    }
    return 0;
}

/* Value a 2-bit code q = 2*b1 + b0 stands for under Eq. 2 with the {-1,+1}
 * bit basis: x = alpha_0 * (2*b0 - 1) + alpha_1 * (2*b1 - 1).
 *   ternary basis  alpha = (1/2, 1/2):  00 -> -1, 01 -> 0, 10 -> 0, 11 -> +1
 *                  (exactly Table 1's codec);
 *   uniform basis  alpha = (1, 2):      00 -> -3, 01 -> -1, 10 -> +1, 11 -> +3. */
static inline int twobit_value(int q, int basis) {
    int b0 = q & 1, b1 = (q >> 1) & 1;
    if (basis == ORACLE_BASIS_TERNARY) return b0 + b1 - 1;
    return (2 * b0 - 1) + 2 * (2 * b1 - 1);
}

/* Eq. 2 with M = K = 2, as the integer dot product it equals.
 * Qw: [M][K], Qa: [N][K] codes in {0,1,2,3}. */
int oracle_twobit_gemm(const int8_t *Qw, const int8_t *Qa, int64_t M, int64_t N, int64_t K,
                       int basis, int32_t *C) {
    int bad = 0;
    for (int64_t i = 0; i < M * K; ++i)
        if (Qw[i] < 0 || Qw[i] > 3) bad = 1;
    for (int64_t i = 0; i < N * K; ++i)
        if (Qa[i] < 0 || Qa[i] > 3) bad = 1;
    if (bad) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int64_t)(twobit_value(Qw[m * K + k], basis) * twobit_value(Qa[n * K + k], basis));
            C[m * N + n] = (int32_t)acc;
        }
    }
    return 0;
}

/* The single high-precision coefficient of the first constraint (Section 3.3),
 * read as one fp32 multiplier per output channel after the integer result, plus
 * an optional bias (batch norm folded, Supplementary S1).
 *   Cf[i][j] = scale[ch] * (float)C[i][j] (+ bias[ch])
 * channel_is_row != 0: ch = i (GEMM, C is [M][N]); else ch = j (NHWC conv output,
 * C is [pixels][Cout]).  One rounding per operation (build with
 * -ffp-contract=off). */
int oracle_scale_epilogue(const int32_t *C, int64_t rows, int64_t cols, int channel_is_row,
                          const float *scale, const float *bias, float *Cf) {
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t j = 0; j < cols; ++j) {
            int64_t ch = channel_is_row ? i : j;
            volatile float prod = scale[ch] * (float)C[i * cols + j];
            float v = prod;
            if (bias) v = v + bias[ch];
            Cf[i * cols + j] = v;
        }
    }
    return 0;
}

/* Eq. 1: binary inner product, bits 0 / 1 standing for -1 / +1.  Bw: [M][K], Ba: [N][K]. */
int oracle_binary_gemm(const int8_t *Bw, const int8_t *Ba, int64_t M, int64_t N, int64_t K, int32_t *C) {
    int bad = 0;
    for (int64_t i = 0; i < M * K; ++i)
        if (Bw[i] != 0 && Bw[i] != 1) bad = 1;
    for (int64_t i = 0; i < N * K; ++i)
        if (Ba[i] != 0 && Ba[i] != 1) bad = 1;
    if (bad) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k) acc += (int64_t)((2 * Bw[m * K + k] - 1) * (2 * Ba[n * K + k] - 1));
            C[m * N + n] = (int32_t)acc;
        }
    }
    return 0;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of OpenMP threads the loops above use from now on (for timing the oracle on one core). */
void oracle_set_num_threads(int n) {
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
