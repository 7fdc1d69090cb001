/*
 * CPU oracle for the micro-rotated FP4 linear-layer path:  Y = Q(X H_b) * Q(W H_b)^T.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain reference that the HIP kernels are checked
 * against.  It shares no code, table or constant with the HIP library and must never be linked or
 * called by the product path.  Only tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What each function follows (paper = arXiv 2509.23202):
 *   orc_hadamard        Sylvester construction of the +-1 Hadamard matrix; the rotation is U = H/sqrt(b)
 *                       (Appendix "Outliers Analysis", proof of Lemma 1; Section 4.1 "Ingredient 3":
 *                       block-diagonal H_k with k x k blocks, k a power of two).
 *   orc_rotate          X H_b with H_b block-diagonal along the reduction (K) axis (Section 4.1,
 *                       Ingredient 3; Section 4.2 item 1).
 *   orc_rotate_dense    X R with R block-diagonal and an arbitrary k x k block given by the caller (Section 4.2
 *                       item 1: any rotation, not just Hadamards, loaded at run time; appendix tables on DCT,
 *                       DST and other transforms).
 *   orc_quantize_mxfp4  MFP format (G=32, E=E2M1, S=E8M0) of Section 2, abs-max scale and round-to-
 *                       nearest of Section 3 (Definition "Scales"), with the scale rounded to a power of
 *                       two by the OCP Microscaling rule  2^(floor(log2 amax) - 2).
 *   orc_quantize_nvfp4  MFP format (G=16, E=E2M1, S=E4M3) plus a per-tensor scale, Section 2 and
 *                       Section 4.1 "Ingredient 1":  Xhat = s_T * s_G * Q(X / (s_T * s_G)).
 *   orc_quantize_*_mse  the same two formats with the group scale chosen to minimise the squared error
 *                       (Section 4.1 "Ingredient 1" objective; "MSE" method of Section 4.2 item 1).
 *   orc_quantize_mxfp4_round43  MXFP4 with the scale rounded in the log domain and re-scaled by 4/3,
 *                       s = (4/3) * 2^clamp(round(log2 s)) (Appendix "MXFP scale fitting", first equation;
 *                       Appendix "Scale quantization analysis").
 *   orc_quantize_mxfp4_fit  MXFP4 with the scale byte re-mapped onto the tensor's own range of scales,
 *                       s = 2^(alpha q + beta) (Appendix "MXFP scale fitting": the modified format MXFP4-dagger);
 *                       orc_quantize_given_scales / orc_dequantize_table: elements against a given table of scale values.
 *   orc_dequantize      the decoding side of the same definitions.
 *   orc_matmul          Y = Ahat * What^T as a plain triple loop in fp64, plus S = |Ahat| * |What|^T.
 *
 * Parity pins (see tests/test_oracle_*.py): every function here is pinned; nothing is "parity unpinned"
 * except the paper's plotted error statistics, which the tests check in direction only.
 *
 * Precision: rotation accumulates in fp64 and rounds once to fp32.  Scale arithmetic for NVFP4 is IEEE
 * binary32, one rounding per written operation (compile with -ffp-contract=off, no fast-math).
 * Element and scale rounding are done by nearest-neighbour search over the decoded grid, ties to the
 * code with an even mantissa bit.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- utilities */

static float bf16_bits_to_float(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---------------------------------------------------------------- Hadamard */

/* Sylvester: H_1 = [1];  H_2n = [[H_n, H_n], [H_n, -H_n]].  H is b*b int8, row-major.
 * Returns 0 on success, -1 if b is not a power of two in [1, 1024]. */
int orc_hadamard(int b, int8_t *H)
{
    if (b < 1 || b > 1024 || (b & (b - 1)) != 0) return -1;
    H[0] = 1;
    for (int n = 1; n < b; n *= 2) {
        /* grow the n*n matrix stored with row stride b into 2n*2n */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                int8_t h = H[i * b + j];
                H[i * b + (j + n)] = h;
                H[(i + n) * b + j] = h;
                H[(i + n) * b + (j + n)] = (int8_t)(-h);
            }
    }
    return 0;
}

/* y[m, j0+c] = (1/sqrt(b)) * sum_r x[m, j0+r] * H[r][c]   for every block j0 = 0, b, 2b, ...
 * x: bf16 bit patterns [M,K] row-major;  y: fp32 [M,K].  fp64 accumulation, ONE rounding to fp32.
 * b == 1 is the identity.  Returns -1 if K % b != 0 or b is invalid. */
int orc_rotate(const uint16_t *x, int64_t M, int64_t K, int b, float *y)
{
    if (b < 1 || b > 1024 || (b & (b - 1)) != 0 || K % b != 0) return -1;
    int8_t *H = (int8_t *)malloc((size_t)b * (size_t)b);
    if (!H) return -2;
    orc_hadamard(b, H);
    const double inv_sqrt_b = 1.0 / sqrt((double)b);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t j0 = 0; j0 < K; j0 += b) {
            for (int c = 0; c < b; ++c) {
                double acc = 0.0;
                for (int r = 0; r < b; ++r)
                    acc += (double)bf16_bits_to_float(x[m * K + j0 + r]) * (double)H[r * b + c];
                y[m * K + j0 + c] = (float)(acc * inv_sqrt_b);
            }
        }
    }
    free(H);
    return 0;
}

/* y = x . blockdiag(R, R, ...) along K with a caller-supplied block R [b,b] (bf16 bit patterns, row-major):
 * y[m, j0 + c] = sum_r x[m, j0 + r] * R[r][c].  fp64 accumulation (every product of two bf16 values is exact in
 * fp64), ONE rounding to fp32.  No normalisation is applied: R carries its own. */
int orc_rotate_dense(const uint16_t *x, int64_t M, int64_t K, int b, const uint16_t *R, float *y)
{
    if (b < 1 || b > 1024 || K % b != 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t j0 = 0; j0 < K; j0 += b) {
            for (int c = 0; c < b; ++c) {
                double acc = 0.0;
                for (int r = 0; r < b; ++r)
                    acc += (double)bf16_bits_to_float(x[m * K + j0 + r]) * (double)bf16_bits_to_float(R[r * b + c]);
                y[m * K + j0 + c] = (float)acc;
            }
        }
    }
    return 0;
}

/* Same rotation applied to an fp64 matrix and kept in fp64 (used by invariance tests only). */
int orc_rotate_f64(const double *x, int64_t M, int64_t K, int b, double *y)
{
    if (b < 1 || b > 1024 || (b & (b - 1)) != 0 || K % b != 0) return -1;
    int8_t *H = (int8_t *)malloc((size_t)b * (size_t)b);
    if (!H) return -2;
    orc_hadamard(b, H);
    const double inv_sqrt_b = 1.0 / sqrt((double)b);
    for (int64_t m = 0; m < M; ++m)
        for (int64_t j0 = 0; j0 < K; j0 += b)
            for (int c = 0; c < b; ++c) {
                double acc = 0.0;
                for (int r = 0; r < b; ++r) acc += x[m * K + j0 + r] * (double)H[r * b + c];
                y[m * K + j0 + c] = acc * inv_sqrt_b;
            }
    free(H);
    return 0;
}

/* ---------------------------------------------------------------- E2M1 elements */

/* Positive E2M1 values in code order (Section 2: 1 sign, 2 exponent, 1 mantissa bit). */
static const double E2M1_GRID[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

double orc_e2m1_decode(uint8_t code)
{
    double v = E2M1_GRID[code & 7];
    return (code & 8) ? -v : v;
}

/* Nearest grid point to v; exact ties go to the code whose mantissa bit (bit 0) is 0;
 * anything beyond the largest value saturates to it.  Sign bit copied from v (so -0.0 and small
 * negatives give 0x8). */
uint8_t orc_e2m1_encode(double v)
{
    uint8_t sign = signbit(v) ? 8 : 0;
    double a = fabs(v);
    if (a >= E2M1_GRID[7]) return (uint8_t)(sign | 7); /* saturation, also keeps huge inputs out of the search */
    int best = 0;
    double best_d = fabs(a - E2M1_GRID[0]);
    for (int c = 1; c < 8; ++c) {
        double d = fabs(a - E2M1_GRID[c]);
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best = c;
            best_d = d;
        }
    }
    return (uint8_t)(sign | best);
}

/* ---------------------------------------------------------------- E8M0 scales */

/* byte e <-> 2^(e-127), e in [0,254]; 255 is NaN and never produced. */
double orc_e8m0_decode(uint8_t e) { return ldexp(1.0, (int)e - 127); }

/* OCP MX rule for a group whose largest magnitude is amax, element format E2M1 (emax = 2):
 * shared exponent = floor(log2(amax)) - 2, clamped to the E8M0 range.  amax == 0 gives byte 0. */
uint8_t orc_e8m0_from_amax(double amax)
{
    if (!(amax > 0.0)) return 0;
    int ex;
    (void)frexp(amax, &ex); /* amax = f * 2^ex with f in [0.5,1)  =>  floor(log2 amax) = ex-1 */
    int E = (ex - 1) - 2;
    int byte = E + 127;
    if (byte < 0) byte = 0;
    if (byte > 254) byte = 254;
    return (uint8_t)byte;
}

/* ---------------------------------------------------------------- E4M3 scales */

/* "fn" flavour: bias 7, no infinities, 0x7F is NaN, largest finite 0x7E = 448; subnormals m * 2^-9. */
double orc_e4m3_decode(uint8_t c)
{
    int e = (c >> 3) & 15, m = c & 7;
    double v = (e == 0) ? ldexp((double)m, -9) : ldexp(1.0 + (double)m / 8.0, e - 7);
    return (c & 0x80) ? -v : v;
}

/* Non-negative input only (a scale).  Nearest of the 127 finite codes 0x00..0x7E, ties to the even
 * code, saturating at 448. */
uint8_t orc_e4m3_encode(double t)
{
    if (!(t > 0.0)) return 0;
    if (t >= 448.0) return 0x7E; /* saturation */
    int best = 0;
    double best_d = t;
    for (int c = 1; c <= 0x7E; ++c) {
        double d = fabs(t - orc_e4m3_decode((uint8_t)c));
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best = c;
            best_d = d;
        }
    }
    return (uint8_t)best;
}

/* ---------------------------------------------------------------- quantizers */

/* MXFP4.  y: fp32 [M,K] (already rotated);  codes: [M,K/2], element k=2j in bits 3:0 of byte j and
 * k=2j+1 in bits 7:4;  scales: [M,K/32] E8M0 bytes.  Returns -1 if K % 32 != 0. */
int orc_quantize_mxfp4(const float *y, int64_t M, int64_t K, uint8_t *codes, uint8_t *scales)
{
    const int G = 32;
    if (K % G != 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t g = 0; g < K / G; ++g) {
            const float *v = y + m * K + g * G;
            double amax = 0.0;
            for (int i = 0; i < G; ++i) {
                double a = fabs((double)v[i]);
                if (a > amax) amax = a;
            }
            uint8_t sb = orc_e8m0_from_amax(amax);
            scales[m * (K / G) + g] = sb;
            double inv = ldexp(1.0, 127 - (int)sb); /* exact power of two */
            for (int i = 0; i < G; i += 2) {
                uint8_t lo = orc_e2m1_encode((double)v[i] * inv);
                uint8_t hi = orc_e2m1_encode((double)v[i + 1] * inv);
                codes[(m * K + g * G + i) / 2] = (uint8_t)(lo | (hi << 4));
            }
        }
    }
    return 0;
}

/* NVFP4 with abs-max scales.  All scale arithmetic is binary32 with one rounding per operation, in
 * exactly this order:
 *     s_T = amax_T / 2688                       (2688 = 6 * 448: largest element times largest scale)
 *     t   = amax_g / (6 * s_T);  c = E4M3(t);  s_G = decode(c)
 *     d   = s_T * s_G;  r = 1 / d;  code_i = E2M1(y_i * r)          (d == 0: all codes 0)
 * y: fp32 [M,K];  codes [M,K/2];  scales [M,K/16] E4M3 bytes;  *s_T_out the tensor scale.
 * If s_T_in is non-NULL its value is used instead of the abs-max one (static tensor scale). */
int orc_quantize_nvfp4(const float *y, int64_t M, int64_t K, const float *s_T_in, uint8_t *codes,
                       uint8_t *scales, float *s_T_out)
{
    const int G = 16;
    if (K % G != 0) return -1;
    float s_T;
    if (s_T_in) {
        s_T = *s_T_in;
    } else {
        float amax_T = 0.0f;
        for (int64_t i = 0; i < M * K; ++i) {
            float a = fabsf(y[i]);
            if (a > amax_T) amax_T = a;
        }
        s_T = amax_T / 2688.0f;
    }
    *s_T_out = s_T;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t g = 0; g < K / G; ++g) {
            const float *v = y + m * K + g * G;
            float amax = 0.0f;
            for (int i = 0; i < G; ++i) {
                float a = fabsf(v[i]);
                if (a > amax) amax = a;
            }
            uint8_t c = 0;
            if (s_T > 0.0f) {
                volatile float six_sT = 6.0f * s_T;
                volatile float t = amax / six_sT;
                c = orc_e4m3_encode((double)t);
            }
            scales[m * (K / G) + g] = c;
            volatile float s_G = (float)orc_e4m3_decode(c);
            volatile float d = s_T * s_G;
            if (d == 0.0f) {
                for (int i = 0; i < G; i += 2) codes[(m * K + g * G + i) / 2] = 0;
                continue;
            }
            volatile float r = 1.0f / d;
            for (int i = 0; i < G; i += 2) {
                volatile float a0 = v[i] * r;
                volatile float a1 = v[i + 1] * r;
                uint8_t lo = orc_e2m1_encode((double)a0);
                uint8_t hi = orc_e2m1_encode((double)a1);
                codes[(m * K + g * G + i) / 2] = (uint8_t)(lo | (hi << 4));
            }
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- MSE scale policy
 * Section 4.2 item 1 names two quantization methods for the fused kernel, abs-max and MSE, without spelling the
 * second out; Section 4.1 "Ingredient 1" states its objective: choose the scales that minimise
 * sum_i (Xhat_i - X_i)^2.  The reading taken here is a per-group search over the scale codes around the abs-max
 * one; a candidate replaces the current choice only if its squared error is strictly smaller, so the order of the
 * candidates decides ties.  MXFP4 (E8M0, one code = a factor 2): abs-max code, one above, one below.  NVFP4 (E4M3,
 * eight codes per octave): abs-max code c0, then c0+1, c0-1, c0+2, c0-2, c0+3, c0+4, c0+5, c0+6, c0+7 -- the
 * minimiser sits either near c0 or about half an octave above it (the scale that puts the group's largest element
 * on the grid value 4 instead of 6), and a brute-force search over every code shows that these windows contain the
 * global minimiser in all but about 1e-4 of the groups of heavy-tailed data (the +-1 window in only half of them for
 * NVFP4).  Errors are exact in fp64 for MXFP4 (power-of-two scales) and accumulated in fp64 for NVFP4.  The NVFP4
 * tensor scale stays the abs-max one (the alternating optimisation over s_T of Ingredient 1 is an offline procedure
 * and not part of the online path). */

static double group_sq_err(const float *v, int G, double scale, double inv, int inv_is_f32, float r32,
                           uint8_t *codes_out)
{
    double err = 0.0;
    for (int i = 0; i < G; ++i) {
        double t;
        if (inv_is_f32) {
            volatile float a = v[i] * r32; /* binary32 product, as the abs-max NVFP4 path rounds it */
            t = (double)a;
        } else {
            t = (double)v[i] * inv; /* exact: power of two */
        }
        const uint8_t c = orc_e2m1_encode(t);
        codes_out[i] = c;
        const double d = (double)v[i] - orc_e2m1_decode(c) * scale;
        err += d * d;
    }
    return err;
}

int orc_quantize_mxfp4_mse(const float *y, int64_t M, int64_t K, uint8_t *codes, uint8_t *scales)
{
    const int G = 32;
    if (K % G != 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t g = 0; g < K / G; ++g) {
            const float *v = y + m * K + g * G;
            double amax = 0.0;
            for (int i = 0; i < G; ++i) {
                double a = fabs((double)v[i]);
                if (a > amax) amax = a;
            }
            const int e0 = (int)orc_e8m0_from_amax(amax);
            const int delta[3] = {0, 1, -1};
            double best_err = 0.0;
            int best_e = e0;
            uint8_t best_codes[32], cand_codes[32];
            for (int k = 0; k < 3; ++k) {
                int e = e0 + delta[k];
                if (e < 0) e = 0;
                if (e > 254) e = 254;
                const double err = group_sq_err(v, G, ldexp(1.0, e - 127), ldexp(1.0, 127 - e), 0, 0.0f, cand_codes);
                if (k == 0 || err < best_err) {
                    best_err = err;
                    best_e = e;
                    memcpy(best_codes, cand_codes, sizeof best_codes);
                }
            }
            scales[m * (K / G) + g] = (uint8_t)best_e;
            for (int i = 0; i < G; i += 2)
                codes[(m * K + g * G + i) / 2] = (uint8_t)(best_codes[i] | (best_codes[i + 1] << 4));
        }
    }
    return 0;
}

int orc_quantize_nvfp4_mse(const float *y, int64_t M, int64_t K, const float *s_T_in, uint8_t *codes,
                           uint8_t *scales, float *s_T_out)
{
    const int G = 16;
    if (K % G != 0) return -1;
    float s_T;
    if (s_T_in) {
        s_T = *s_T_in;
    } else {
        float amax_T = 0.0f;
        for (int64_t i = 0; i < M * K; ++i) {
            float a = fabsf(y[i]);
            if (a > amax_T) amax_T = a;
        }
        s_T = amax_T / 2688.0f;
    }
    *s_T_out = s_T;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t g = 0; g < K / G; ++g) {
            const float *v = y + m * K + g * G;
            float amax = 0.0f;
            for (int i = 0; i < G; ++i) {
                float a = fabsf(v[i]);
                if (a > amax) amax = a;
            }
            int c0 = 0;
            if (s_T > 0.0f) {
                volatile float six_sT = 6.0f * s_T;
                volatile float t = amax / six_sT;
                c0 = (int)orc_e4m3_encode((double)t);
            }
            const int delta[10] = {0, 1, -1, 2, -2, 3, 4, 5, 6, 7};
            double best_err = 0.0;
            int best_c = c0;
            uint8_t best_codes[16], cand_codes[16];
            for (int k = 0; k < 10; ++k) {
                int c = c0 + delta[k];
                if (c < 0) c = 0;
                if (c > 0x7e) c = 0x7e;
                volatile float s_G = (float)orc_e4m3_decode((uint8_t)c);
                volatile float d = s_T * s_G;
                double err;
                if (d == 0.0f) {
                    err = 0.0;
                    for (int i = 0; i < G; ++i) {
                        cand_codes[i] = 0;
                        err += (double)v[i] * (double)v[i];
                    }
                } else {
                    volatile float r = 1.0f / d;
                    err = group_sq_err(v, G, (double)d, 0.0, 1, r, cand_codes);
                }
                if (k == 0 || err < best_err) {
                    best_err = err;
                    best_c = c;
                    memcpy(best_codes, cand_codes, sizeof best_codes);
                }
            }
            scales[m * (K / G) + g] = (uint8_t)best_c;
            for (int i = 0; i < G; i += 2)
                codes[(m * K + g * G + i) / 2] = (uint8_t)(best_codes[i] | (best_codes[i + 1] << 4));
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- alternating optimisation of the NVFP4 scales
 * Section 4.1 "Ingredient 1": minimise sum_i (Xhat_i - X_i)^2 over the tensor scale s_T and the group scales
 * s_G1..s_Gk "by alternating optimization over the block scales and the per-tensor scale".  The paper gives no
 * further detail; the reading taken here:
 *     start:        s_T = amax_T / 2688 (the abs-max tensor scale)
 *     block step:   with s_T fixed, every group takes the E4M3 code of the squared-error search above
 *                   (orc_quantize_nvfp4_mse) and its elements are rounded to nearest
 *     tensor step:  with codes and group scales fixed, Xhat_i = s_T * v_i with v_i = s_G(i) * E2M1(code_i), and the
 *                   minimiser is the least-squares factor  s_T = sum_i X_i v_i / sum_i v_i^2  (sums in fp64 in index
 *                   order, quotient rounded once to binary32); if the denominator or the numerator is not positive
 *                   s_T is kept and the iteration stops
 *     `rounds` times (block step, tensor step), then one last block step so that the returned codes are the
 *     round-to-nearest codes of the returned scales.
 * s_T_trace (may be NULL) receives the rounds + 1 tensor scales in order. */
int orc_quantize_nvfp4_mse_alt(const float *y, int64_t M, int64_t K, int rounds, uint8_t *codes, uint8_t *scales,
                               float *s_T_out, float *s_T_trace)
{
    const int G = 16;
    if (K % G != 0 || rounds < 0) return -1;
    float s_T = 0.0f;
    if (orc_quantize_nvfp4_mse(y, M, K, NULL, codes, scales, &s_T) != 0) return -1;
    if (s_T_trace) s_T_trace[0] = s_T;
    for (int r = 0; r < rounds; ++r) {
        double num = 0.0, den = 0.0;
        for (int64_t i = 0; i < M * K; ++i) {
            const uint8_t byte = codes[i / 2];
            const uint8_t code = (i & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 15);
            const double v = orc_e2m1_decode(code) * orc_e4m3_decode(scales[i / G]);
            num += (double)y[i] * v;
            den += v * v;
        }
        if (den > 0.0 && num > 0.0) {
            s_T = (float)(num / den);
            float unused;
            if (orc_quantize_nvfp4_mse(y, M, K, &s_T, codes, scales, &unused) != 0) return -1;
        }
        if (s_T_trace) s_T_trace[r + 1] = s_T;
    }
    *s_T_out = s_T;
    return 0;
}

/* ---------------------------------------------------------------- rounded, 4/3-rescaled E8M0 scale
 * Appendix "MXFP scale fitting", first equation (and Appendix "Scale quantization analysis"): the scale of a group
 * is quantized as  (4/3) * 2^clamp(round(log2 s)).  Readings taken here: s is the ideal abs-max scale amax / 6 (the
 * largest element lands on the largest grid value, Section 3 "Scales"); round is to the nearest integer (log2 s is
 * never a half-integer for a binary floating-point s); the exponent is clamped to what an E8M0 byte can hold,
 * [-127, 127] (the equation's -128 has no byte).  The byte stores the exponent only; the constant 4/3 belongs to
 * the whole tensor and is applied where the tensor is decoded (orc_dequantize's s_T).  Elements are rounded to the
 * nearest E2M1 value of  v / ((4/3) 2^k) = 0.75 v 2^-k, which is exact in fp64 for an fp32 v.
 * amax == 0 gives byte 0. */
uint8_t orc_e8m0_round43_from_amax(double amax)
{
    if (!(amax > 0.0)) return 0;
    const double l = log2(amax / 6.0);
    int k = (int)floor(l + 0.5);
    if (k < -127) k = -127;
    if (k > 127) k = 127;
    return (uint8_t)(k + 127);
}

int orc_quantize_mxfp4_round43(const float *y, int64_t M, int64_t K, uint8_t *codes, uint8_t *scales)
{
    const int G = 32;
    if (K % G != 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t g = 0; g < K / G; ++g) {
            const float *v = y + m * K + g * G;
            double amax = 0.0;
            for (int i = 0; i < G; ++i) {
                double a = fabs((double)v[i]);
                if (a > amax) amax = a;
            }
            const uint8_t sb = orc_e8m0_round43_from_amax(amax);
            scales[m * (K / G) + g] = sb;
            const double inv = ldexp(0.75, 127 - (int)sb); /* 1 / ((4/3) 2^k) */
            for (int i = 0; i < G; i += 2) {
                uint8_t lo = orc_e2m1_encode((double)v[i] * inv);
                uint8_t hi = orc_e2m1_encode((double)v[i + 1] * inv);
                codes[(m * K + g * G + i) / 2] = (uint8_t)(lo | (hi << 4));
            }
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- scale byte fitted to the tensor's range of scales
 * Appendix "MXFP scale fitting": the 256 codes of the scale byte are spread over the range of scales that the tensor
 * actually has instead of over 2^-127 .. 2^127.  With s the ideal abs-max scale of a group (amax / 6, as in the first
 * equation of that appendix) and s_min, s_max its smallest and largest value over the tensor,
 *     q = clamp(round(255 (log2 s - log2 s_min) / (log2 s_max - log2 s_min)), 0, 255)
 *     s_hat = 2^(alpha q + beta),   alpha = (log2 s_max - log2 s_min) / 255,   beta = log2 s_min.
 * Readings taken here (the appendix prints the second equation without the division by 255 in the exponent; it is
 * needed for q = 255 to decode to s_max, and the third equation, s = 2^(alpha q + beta) with alpha in (0, 1), says the
 * same): groups that are all zero take no part in s_min, get q = 0 and zero codes; a tensor with a single distinct
 * scale has alpha = 0; an all-zero tensor has alpha = beta = 0.  Elements are rounded to the nearest E2M1 value of
 * v / s_hat (saturating at 6: s_hat can be below s by up to half a step of the grid, 2^(alpha/2)).
 * If ab_in is non-NULL its (alpha, beta) are used instead of the fitted ones (a layer whose weights and activations must
 * share alpha, last paragraph of the appendix) and q is clamped to the byte.
 * y: fp32 [M,K];  codes [M,K/2];  q [M,K/32];  ab_out[2] = (alpha, beta);  table[256] = s_hat(0..255).  All fp64. */
int orc_quantize_mxfp4_fit(const float *y, int64_t M, int64_t K, const double *ab_in, uint8_t *codes, uint8_t *q,
                           double *ab_out, double *table)
{
    const int G = 32;
    if (K % G != 0) return -1;
    const int64_t NG = M * (K / G);
    double *amax = (double *)malloc(sizeof(double) * (size_t)(NG > 0 ? NG : 1));
    if (!amax) return -2;
    double lo = INFINITY, hi = 0.0;
    for (int64_t g = 0; g < NG; ++g) {
        double a = 0.0;
        for (int i = 0; i < G; ++i) {
            double t = fabs((double)y[g * G + i]);
            if (t > a) a = t;
        }
        amax[g] = a;
        if (a > 0.0 && a < lo) lo = a;
        if (a > hi) hi = a;
    }
    double alpha = 0.0, beta = 0.0;
    if (ab_in) {
        alpha = ab_in[0];
        beta = ab_in[1];
    } else if (hi > 0.0) {
        beta = log2(lo / 6.0);
        alpha = (log2(hi / 6.0) - beta) / 255.0;
    }
    ab_out[0] = alpha;
    ab_out[1] = beta;
    for (int c = 0; c < 256; ++c) table[c] = exp2(alpha * c + beta);
    for (int64_t g = 0; g < NG; ++g) {
        int c = 0;
        if (amax[g] > 0.0 && alpha > 0.0) {
            const double t = (log2(amax[g] / 6.0) - beta) / alpha;
            c = (int)floor(t + 0.5);
            if (c < 0) c = 0;
            if (c > 255) c = 255;
        }
        q[g] = (uint8_t)c;
        for (int i = 0; i < G; i += 2) {
            uint8_t l = 0, h = 0;
            if (amax[g] > 0.0) {
                l = orc_e2m1_encode((double)y[g * G + i] / table[c]);
                h = orc_e2m1_encode((double)y[g * G + i + 1] / table[c]);
            }
            codes[(g * G + i) / 2] = (uint8_t)(l | (h << 4));
        }
    }
    free(amax);
    return 0;
}

/* Elements of [M,K] against GIVEN scales: group g uses the binary32 value table[q[g]], and the arithmetic is the binary32
 * chain of orc_quantize_nvfp4 (r = 1 / d rounded, y * r rounded, then the nearest E2M1 value); a group whose values are
 * all zero gets zero codes.  G = 32. */
int orc_quantize_given_scales(const float *y, int64_t M, int64_t K, const uint8_t *q, const float *table, uint8_t *codes)
{
    const int G = 32;
    if (K % G != 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < M * (K / G); ++g) {
        const float *v = y + g * G;
        float amax = 0.0f;
        for (int i = 0; i < G; ++i) {
            float a = fabsf(v[i]);
            if (a > amax) amax = a;
        }
        volatile float d = table[q[g]];
        if (amax == 0.0f || d == 0.0f) {
            for (int i = 0; i < G; i += 2) codes[(g * G + i) / 2] = 0;
            continue;
        }
        volatile float r = 1.0f / d;
        for (int i = 0; i < G; i += 2) {
            volatile float a0 = v[i] * r;
            volatile float a1 = v[i + 1] * r;
            codes[(g * G + i) / 2] = (uint8_t)(orc_e2m1_encode((double)a0) | (orc_e2m1_encode((double)a1) << 4));
        }
    }
    return 0;
}

/* out[m,k] = E2M1(code) * table[q of the group]  (G = 32; table in fp64). */
int orc_dequantize_table(const uint8_t *codes, const uint8_t *q, const double *table, int64_t M, int64_t K, double *out)
{
    const int G = 32;
    if (K % G != 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            uint8_t byte = codes[(m * K + k) / 2];
            uint8_t code = (k & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 15);
            out[m * K + k] = orc_e2m1_decode(code) * table[q[m * (K / G) + k / G]];
        }
    return 0;
}

/* fmt 0 = MXFP4 (G=32, E8M0), fmt 1 = NVFP4 (G=16, E4M3); both times the tensor-level factor s_T (1 for plain
 * MXFP4, 4/3 for the re-scaled E8M0 rule, the tensor scale for NVFP4).  out: fp64 [M,K]. */
int orc_dequantize(const uint8_t *codes, const uint8_t *scales, double s_T, int fmt, int64_t M,
                   int64_t K, double *out)
{
    const int G = (fmt == 0) ? 32 : 16;
    if (fmt != 0 && fmt != 1) return -1;
    if (K % G != 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            uint8_t byte = codes[(m * K + k) / 2];
            uint8_t code = (k & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 15);
            uint8_t sb = scales[m * (K / G) + k / G];
            double s = ((fmt == 0) ? orc_e8m0_decode(sb) : orc_e4m3_decode(sb)) * s_T;
            out[m * K + k] = orc_e2m1_decode(code) * s;
        }
    return 0;
}

/* ---------------------------------------------------------------- contraction */

/* Y[m,n] = sum_k A[m,k] * W[n,k];  S[m,n] = sum_k |A[m,k]| * |W[n,k]|   (S may be NULL).
 * A: [M,K], W: [N,K], both fp64 row-major.  Plain loops, k innermost, ascending. */
void orc_matmul(const double *A, const double *W, int64_t M, int64_t N, int64_t K, double *Y, double *S)
{
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, accs = 0.0;
            const double *a = A + m * K, *w = W + n * K;
            for (int64_t k = 0; k < K; ++k) {
                double p = a[k] * w[k];
                acc += p;
                accs += fabs(p);
            }
            Y[m * N + n] = acc;
            if (S) S[m * N + n] = accs;
        }
}
