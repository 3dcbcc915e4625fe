/*
 * dma_oracle.c -- CPU oracle for Diagonal-Tiled Mixed-Precision Attention (DMA).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, step-by-step statement of what the
 * method computes.  It is used by the tests, by the smoke check and by the benchmark's CPU
 * baseline leg, and by nothing else; the GPU library never links, loads or calls it, and it
 * shares no code, table or header with the GPU path.
 *
 * Everything after quantization is done in double.  Each function cites the passage of the
 * paper it follows (section / algorithm / equation / table).
 *
 * Formats: 0 = unquantized bf16, 1 = MXFP8 with E4M3 elements, 2 = MXFP4 with E2M1 elements,
 * 3 = MXFP8 with E5M2 elements; MX block = 32 consecutive elements along the head dimension with one E8M0 scale byte
 * (Table "Comparison of representative MXFP data formats"; Sec. 3.1).
 *
 * Readings taken where the paper is silent or inconsistent are listed at each place they are
 * used, prefixed "Reading:".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_FMT_BF16 0
#define ORACLE_FMT_E4M3 1
#define ORACLE_FMT_E2M1 2
#define ORACLE_FMT_E5M2 3

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_MEM (-2)

/* ------------------------------------------------------------------------------------------ */
/* bf16 <-> binary32 / double                                                                 */
/* ------------------------------------------------------------------------------------------ */

/* bf16 is the upper half of a binary32 word, so widening is exact. */
float oracle_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Round a double to the nearest bf16 (8 significand bits incl. the hidden one), ties to even,
 * in ONE rounding step (no detour through binary32).  Returns the value as a double.
 * Used for the probabilities that enter the P*V product (Reading: P is rounded to the 16-bit
 * type of V before the second product, the flash-attention idiom; Alg. 1 keeps V in 16 bit). */
double oracle_round_to_bf16(double p)
{
    if (p == 0.0 || isnan(p) || isinf(p)) return p;
    int ex;
    (void)frexp(p, &ex);              /* |p| = f * 2^ex, f in [0.5, 1)  ->  floor(log2|p|) = ex-1 */
    int quantum = (ex - 1) - 7;       /* spacing of bf16 numbers in [2^(ex-1), 2^ex) is 2^(ex-1-7) */
    if (quantum < -133) quantum = -133; /* bf16 subnormals: fixed spacing 2^-133 */
    double scaled = ldexp(p, -quantum);
    double r = nearbyint(scaled);     /* default rounding mode = to nearest, ties to even */
    return ldexp(r, quantum);
}

/* ------------------------------------------------------------------------------------------ */
/* Element encoders / decoders                                                                */
/* ------------------------------------------------------------------------------------------ */

/* E2M1 decode: bit layout (S<<3)|(E<<1)|M with exponent bias 1 (Alg. 3, Step 4.4).
 * E = 0 is subnormal: value M * 0.5.  Otherwise (1 + M/2) * 2^(E-1).
 * Magnitudes by code 0..7: 0, 0.5, 1, 1.5, 2, 3, 4, 6. */
double oracle_e2m1_decode(uint8_t code)
{
    int s = (code >> 3) & 1, e = (code >> 1) & 3, m = code & 1;
    double a = (e == 0) ? 0.5 * m : ldexp(1.0 + 0.5 * m, e - 1);
    return s ? -a : a;
}

/* E2M1 encode of a value already scaled and clamped to [-6, 6] (Alg. 2 Step 4; Alg. 3).
 * Reading: the printed mantissa rule is not a complete rounding (no carry into the exponent,
 * and its subnormal threshold is inconsistent with the text); the text states the intent:
 * round to nearest with ties to the even mantissa (its example: 5 -> 4), thresholds strict.
 * This is that rounding, written out.  The sign bit is the sign bit of the input, also for
 * results that round to zero (Alg. 3 Step 4.1 takes the sign first). */
uint8_t oracle_e2m1_encode(double y, int negative)
{
    double a = fabs(y);
    int mag;
    if (a < 1.0) {
        /* subnormal range and the step up to 1.0: grid 0, 0.5, 1.0  = codes 0, 1, 2 */
        mag = (int)nearbyint(2.0 * a);
    } else {
        int ex;
        (void)frexp(a, &ex);
        int e = ex - 1;                                   /* floor(log2 a): 0, 1 or 2 */
        int m = (int)nearbyint(2.0 * (ldexp(a, -e) - 1.0)); /* 0, 1, or 2 (= carry) */
        if (m == 2) { e += 1; m = 0; }
        mag = ((e + 1) << 1) | m;
    }
    if (mag > 7) mag = 7;
    return (uint8_t)((negative ? 8 : 0) | mag);
}

/* E4M3 decode (OCP variant: bias 7, exponent field 15 is an ordinary binade, no infinities;
 * Sec. 4.2 "Compute shared scale": e_max = 8).  E = 0: M * 2^-9.  Else (1 + M/8) * 2^(E-7). */
double oracle_e4m3_decode(uint8_t code)
{
    int s = (code >> 7) & 1, e = (code >> 3) & 15, m = code & 7;
    double a = (e == 0) ? ldexp((double)m, -9) : ldexp(1.0 + m / 8.0, e - 7);
    return s ? -a : a;
}

/* E4M3 encode of a value already scaled and clamped to [-448, 448] (Alg. 2 Step 6).
 * Reading: the algorithm shows only the clamp; the element conversion is round to nearest,
 * ties to even, with subnormals, as for the 4-bit format.  0x7F / 0xFF are never produced. */
uint8_t oracle_e4m3_encode(double y, int negative)
{
    double a = fabs(y);
    int mag;
    if (a < ldexp(1.0, -6)) {
        mag = (int)nearbyint(ldexp(a, 9));                /* 0..8; 8 is the first normal */
    } else {
        int ex;
        (void)frexp(a, &ex);
        int e = ex - 1;                                   /* -6 .. 8 */
        int m = (int)nearbyint(8.0 * (ldexp(a, -e) - 1.0)); /* 0..8 (8 = carry) */
        if (m == 8) { e += 1; m = 0; }
        mag = ((e + 7) << 3) | m;
    }
    if (mag > 0x7E) mag = 0x7E;
    return (uint8_t)((negative ? 0x80 : 0) | mag);
}

/* E5M2 decode (Table of MX formats; Sec. 4.2 "Compute shared scale": e_max = 15, i.e. exponent field 30 with
 * bias 15; field 31 is reserved for infinities and NaN).  E = 0: M * 2^-16.  Else (1 + M/4) * 2^(E-15).
 * Largest finite magnitude 1.75 * 2^15 = 57344 = code 0x7B. */
double oracle_e5m2_decode(uint8_t code)
{
    int s = (code >> 7) & 1, e = (code >> 2) & 31, m = code & 3;
    double a = (e == 0) ? ldexp((double)m, -16) : ldexp(1.0 + m / 4.0, e - 15);
    return s ? -a : a;
}

/* E5M2 encode of a value already scaled and clamped to [-57344, 57344] (Alg. 2 Step 6 with the
 * E5M2 bounds).  Reading: as for E4M3, round to nearest, ties to even, with subnormals; the
 * reserved codes (exponent field 31) are never produced. */
uint8_t oracle_e5m2_encode(double y, int negative)
{
    double a = fabs(y);
    int mag;
    if (a < ldexp(1.0, -14)) {
        mag = (int)nearbyint(ldexp(a, 16));               /* 0..4; 4 is the first normal */
    } else {
        int ex;
        (void)frexp(a, &ex);
        int e = ex - 1;                                   /* -14 .. 15 */
        int m = (int)nearbyint(4.0 * (ldexp(a, -e) - 1.0)); /* 0..4 (4 = carry) */
        if (m == 4) { e += 1; m = 0; }
        mag = ((e + 15) << 2) | m;
    }
    if (mag > 0x7B) mag = 0x7B;
    return (uint8_t)((negative ? 0x80 : 0) | mag);
}

/* Exponent of the largest normal number of the element format (Sec. 4.2: 8 for E4M3; for E2M1
 * the largest normal is 6 = 1.5 * 2^2, so 2).  Reading: the MXFP4 copy uses the same E8M0 rule
 * as the MXFP8 copy (text of "Compute shared scale"), not the max/6 rule of Alg. 2 Step 3,
 * which is the NVFP4 flavour. */
static int fmt_emax(int fmt) { return fmt == ORACLE_FMT_E2M1 ? 2 : fmt == ORACLE_FMT_E5M2 ? 15 : 8; }
static double fmt_maxval(int fmt) { return fmt == ORACLE_FMT_E2M1 ? 6.0 : fmt == ORACLE_FMT_E5M2 ? 57344.0 : 448.0; }
static int fmt_is_mx(int fmt) { return fmt == ORACLE_FMT_E4M3 || fmt == ORACLE_FMT_E2M1 || fmt == ORACLE_FMT_E5M2; }

/* E8M0 scale byte of a block whose absolute maximum (a binary32 value) is amax
 * (Alg. 2 Step 6: S_shared = floor(log2 amax) - e_max;  Step 7: clamp(S_shared + 127, 0, 254)).
 * amax = 0 gives log2 = -inf, which the clamp maps to 0. */
uint8_t oracle_e8m0_from_amax(float amax, int fmt)
{
    if (!(amax > 0.0f)) return 0;
    int ex;
    (void)frexp((double)amax, &ex);
    long shared = (long)(ex - 1) - fmt_emax(fmt);   /* floor(log2 amax) - e_max */
    long biased = shared + 127;
    if (biased < 0) biased = 0;
    if (biased > 254) biased = 254;
    return (uint8_t)biased;
}

/* The query pre-scale log2(e)/sqrt(D) (Alg. 2 Step 1), as the binary32 constant.
 * Reading: the product x * c is ONE binary32 multiplication, kept in binary32. */
float oracle_query_prescale(int D)
{
    return (float)(1.4426950408889634074 / sqrt((double)D));
}

/* ------------------------------------------------------------------------------------------ */
/* MX quantization of a [rows, D] bf16 matrix (Alg. 2, Steps 1 and 3-7)                       */
/* ------------------------------------------------------------------------------------------ */

/* The per-token scale of Alg. 2 Step 2 for a row whose absolute maximum (after Step 1) is amax:
 * S_q = amax / (448 * 6), and the factor the row is multiplied by, 1 / S_q.
 * Reading: both are ONE binary32 division each (amax / 2688 and 2688 / amax), and X / S_q is the
 * binary32 product X * (2688 / amax).  Rows with amax below 2^-100 (zero rows included) are left
 * alone (S_q = 1): their reciprocal would overflow. */
void oracle_token_scale(float amax, float *s_q, float *inv_s_q)
{
    if (!(amax >= 0x1p-100f)) { *s_q = 1.0f; *inv_s_q = 1.0f; return; }
    volatile float a = amax / 2688.0f, b = 2688.0f / amax;
    *s_q = a;
    *inv_s_q = b;
}

/* Quantize one row.  codes: D bytes (E4M3, E5M2) or D/2 bytes (E2M1, element 2t in the low nibble
 * and 2t+1 in the high nibble: Alg. 2 Step 5 and "Packing").  scales: D/32 bytes.
 * per_token == 0.  Reading: the per-token scale S_q of Alg. 2 Step 2 is 1 on the default path (it
 * exists to fit the E4M3-typed scale of NVFP4; an E8M0 scale already spans the binary32 range,
 * Sec. 3.1).
 * per_token != 0: Alg. 2 Step 2 as printed: the row is divided by S_q = max_D|X| / (448 * 6) before
 * the shared scales are formed; *token_scale receives S_q (the dequantized row is decode * S_q).
 * amax_in >= 0 (with per_token != 0): the maximum is not the row's own but that of the group of rows
 * it belongs to (Sec. 5.3 names per-block and per-tensor granularities of this scale), given by the
 * caller (oracle_group_amax). */
static void quantize_row(const uint16_t *x, int D, int fmt, int is_query, int per_token, float amax_in,
                         uint8_t *codes, uint8_t *scales, float *token_scale)
{
    const float c = oracle_query_prescale(D);
    float xs[32];
    float s_q = 1.0f, inv_s_q = 1.0f;
    if (per_token) {
        float rmax = 0.0f;
        for (int d = 0; d < D; ++d) {
            float v = oracle_bf16_to_f32(x[d]);
            if (is_query) {
                volatile float prod = v * c;
                v = prod;
            }
            if (fabsf(v) > rmax) rmax = fabsf(v);
        }
        if (amax_in >= 0.0f) rmax = amax_in;
        oracle_token_scale(rmax, &s_q, &inv_s_q);
    }
    if (token_scale) *token_scale = s_q;
    for (int blk = 0; blk < D / 32; ++blk) {
        float amax = 0.0f;
        for (int t = 0; t < 32; ++t) {
            float v = oracle_bf16_to_f32(x[blk * 32 + t]);
            if (is_query) {
                volatile float prod = v * c;     /* one binary32 multiply, rounded once */
                v = prod;
            }
            if (per_token) {
                volatile float prod = v * inv_s_q;   /* X / S_q, one binary32 multiply */
                v = prod;
            }
            xs[t] = v;
            float av = fabsf(v);
            if (av > amax) amax = av;
        }
        uint8_t sc = oracle_e8m0_from_amax(amax, fmt);
        scales[blk] = sc;
        const double u = fmt_maxval(fmt);
        for (int t = 0; t < 32; ++t) {
            int neg = signbit(xs[t]) ? 1 : 0;
            double y = ldexp((double)xs[t], 127 - (int)sc);     /* x / 2^S_shared, exact */
            if (y > u) y = u;                                   /* clamp(., l, u) */
            if (y < -u) y = -u;
            int d = blk * 32 + t;
            if (fmt == ORACLE_FMT_E2M1) {
                uint8_t cd = oracle_e2m1_encode(y, neg);
                if (d & 1) codes[d >> 1] = (uint8_t)(codes[d >> 1] | (cd << 4));
                else       codes[d >> 1] = cd;
            } else if (fmt == ORACLE_FMT_E5M2) {
                codes[d] = oracle_e5m2_encode(y, neg);
            } else {
                codes[d] = oracle_e4m3_encode(y, neg);
            }
        }
    }
}

/* Maximum magnitude (after the query pre-scale if is_query) of the group each row belongs to, for
 * Alg. 2 Step 2 at the granularities Sec. 5.3 names.  x: [n_mat, S, D] bf16; out: [n_mat * S].
 * gran 1: the row itself (per-token); 2: blocks of block_rows consecutive rows of one [S, D] matrix,
 * starting at multiples of block_rows (per-block; the last block of a matrix may be shorter);
 * 3: all of x (per-tensor).
 * Reading: the paper names the granularities without defining the groups; a block is taken to be the
 * rows of one attention tile of one head, the tensor everything passed to the call. */
int oracle_group_amax(const uint16_t *x, int64_t n_mat, int64_t S, int D, int is_query, int gran,
                      int64_t block_rows, float *out)
{
    if (!x || !out || n_mat <= 0 || S <= 0 || D <= 0 || gran < 1 || gran > 3) return ORACLE_ERR_ARG;
    if (gran == 2 && block_rows <= 0) return ORACLE_ERR_ARG;
    const float c = oracle_query_prescale(D);
    const int64_t rows = n_mat * S;
    for (int64_t r = 0; r < rows; ++r) {
        float rmax = 0.0f;
        for (int d = 0; d < D; ++d) {
            float v = oracle_bf16_to_f32(x[r * D + d]);
            if (is_query) {
                volatile float prod = v * c;
                v = prod;
            }
            if (fabsf(v) > rmax) rmax = fabsf(v);
        }
        out[r] = rmax;
    }
    if (gran == 2) {
        for (int64_t mtx = 0; mtx < n_mat; ++mtx)
            for (int64_t r0 = 0; r0 < S; r0 += block_rows) {
                const int64_t r1 = (r0 + block_rows < S) ? r0 + block_rows : S;
                float g = 0.0f;
                for (int64_t r = r0; r < r1; ++r)
                    if (out[mtx * S + r] > g) g = out[mtx * S + r];
                for (int64_t r = r0; r < r1; ++r) out[mtx * S + r] = g;
            }
    } else if (gran == 3) {
        float g = 0.0f;
        for (int64_t r = 0; r < rows; ++r)
            if (out[r] > g) g = out[r];
        for (int64_t r = 0; r < rows; ++r) out[r] = g;
    }
    return ORACLE_OK;
}

/* token_scales: NULL = Step 2 skipped (S_q = 1); else [rows] binary32, receives S_q of every row.
 * amax_in: NULL = the scale of a row comes from its own maximum; else [rows], the maximum of the row's group. */
int oracle_mx_quantize_grouped(const uint16_t *x, int64_t rows, int D, int fmt, int is_query, const float *amax_in,
                               uint8_t *codes, uint8_t *scales, float *token_scales)
{
    if (!x || !codes || !scales || !token_scales || !amax_in || rows < 0 || D <= 0 || D % 32 != 0) return ORACLE_ERR_ARG;
    if (!fmt_is_mx(fmt)) return ORACLE_ERR_ARG;
    const int64_t cb = (fmt == ORACLE_FMT_E2M1) ? D / 2 : D;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        quantize_row(x + r * D, D, fmt, is_query, 1, amax_in[r], codes + r * cb, scales + r * (D / 32), token_scales + r);
    return ORACLE_OK;
}

int oracle_mx_quantize_ex(const uint16_t *x, int64_t rows, int D, int fmt, int is_query,
                          uint8_t *codes, uint8_t *scales, float *token_scales)
{
    if (!x || !codes || !scales || rows < 0 || D <= 0 || D % 32 != 0) return ORACLE_ERR_ARG;
    if (!fmt_is_mx(fmt)) return ORACLE_ERR_ARG;
    const int64_t cb = (fmt == ORACLE_FMT_E2M1) ? D / 2 : D;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        quantize_row(x + r * D, D, fmt, is_query, token_scales != NULL, -1.0f, codes + r * cb, scales + r * (D / 32),
                     token_scales ? token_scales + r : NULL);
    return ORACLE_OK;
}

int oracle_mx_quantize(const uint16_t *x, int64_t rows, int D, int fmt, int is_query,
                       uint8_t *codes, uint8_t *scales)
{
    return oracle_mx_quantize_ex(x, rows, D, fmt, is_query, codes, scales, NULL);
}

/* Decode codes + scales back to real values: element * 2^(scale - 127), exact in double. */
int oracle_mx_dequantize(const uint8_t *codes, const uint8_t *scales, int64_t rows, int D, int fmt,
                         double *out)
{
    if (!codes || !scales || !out || rows < 0 || D <= 0 || D % 32 != 0) return ORACLE_ERR_ARG;
    if (!fmt_is_mx(fmt)) return ORACLE_ERR_ARG;
    const int64_t cb = (fmt == ORACLE_FMT_E2M1) ? D / 2 : D;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int d = 0; d < D; ++d) {
            int sc = scales[r * (D / 32) + d / 32];
            double e;
            if (fmt == ORACLE_FMT_E2M1) {
                uint8_t b = codes[r * cb + (d >> 1)];
                e = oracle_e2m1_decode((d & 1) ? (uint8_t)(b >> 4) : (uint8_t)(b & 15));
            } else if (fmt == ORACLE_FMT_E5M2) {
                e = oracle_e5m2_decode(codes[r * cb + d]);
            } else {
                e = oracle_e4m3_decode(codes[r * cb + d]);
            }
            out[r * D + d] = ldexp(e, sc - 127);
        }
    }
    return ORACLE_OK;
}

/* What a row looks like to the score product in format fmt, as doubles:
 * quantized formats: quantize then decode; bf16: the values themselves (the softmax factor is
 * then applied to the score, see score_scale()). */
static void row_as_seen(const uint16_t *x, int D, int fmt, int is_query, int per_token, float amax_in, double *out)
{
    if (fmt == ORACLE_FMT_BF16) {
        for (int d = 0; d < D; ++d) out[d] = (double)oracle_bf16_to_f32(x[d]);
        return;
    }
    uint8_t codes[1024];
    uint8_t scales[64];
    float s_q = 1.0f;
    memset(codes, 0, sizeof codes);
    quantize_row(x, D, fmt, is_query, per_token, amax_in, codes, scales, &s_q);
    oracle_mx_dequantize(codes, scales, 1, D, fmt, out);
    if (per_token)
        for (int d = 0; d < D; ++d) out[d] *= (double)s_q;       /* the dequantization multiplier of Step 2 */
}

/* ------------------------------------------------------------------------------------------ */
/* MX-format P V (an extension beyond Alg. 1, which keeps V and P in 16 bit)                     */
/* ------------------------------------------------------------------------------------------ */
/* The second product contracts over keys, so its MX blocks run along the key axis: 32 consecutive
 * keys (aligned to multiples of 32) of one head-dimension column of V, and 32 consecutive keys of
 * one query row of P, each with one E8M0 scale byte and E4M3 elements, quantized by the rule of
 * Alg. 2 Steps 6-7 (shared scale from the block maximum with e_max = 8, clamp to +-448, round to
 * nearest even).  Keys at or beyond S count as zeros. */

/* One block of n <= 32 real values: its scale byte and what the block looks like after
 * quantize + decode.  x holds binary32-representable values or probabilities in [0, 1].
 * shift (0 except for the alternatives a parity test asks for, see row_alts) is added to the
 * scale byte the rule gives before the byte is clamped. */
static int block_e4m3_as_seen(const double *x, int n, int shift, double *seen)
{
    double amax = 0.0;
    for (int t = 0; t < n; ++t)
        if (fabs(x[t]) > amax) amax = fabs(x[t]);
    long biased = 0;
    if (amax > 0.0) {
        int ex;
        (void)frexp(amax, &ex);
        biased = (long)(ex - 1) - 8 + 127 + shift;  /* floor(log2 amax) - e_max, biased */
        if (biased < 0) biased = 0;
        if (biased > 254) biased = 254;
    }
    for (int t = 0; t < n; ++t) {
        double y = ldexp(x[t], 127 - (int)biased);
        if (y > 448.0) y = 448.0;
        if (y < -448.0) y = -448.0;
        seen[t] = ldexp(oracle_e4m3_decode(oracle_e4m3_encode(y, signbit(x[t]) ? 1 : 0)), (int)biased - 127);
    }
    return (int)biased;
}

/* V of one kv head as the MX-format P V product sees it: v [S, D] bf16 -> seen [n, D] doubles for the
 * keys 0 .. n-1 (n a multiple of 32 or n = S; blocks that reach past S are padded with zeros). */
int oracle_values_as_seen_mxfp8(const uint16_t *v, int64_t S, int D, int64_t n, double *seen, uint8_t *scales)
{
    if (!v || !seen || S <= 0 || D <= 0 || n <= 0 || n > ((S + 31) / 32) * 32) return ORACLE_ERR_ARG;
    const int64_t nblk = (n + 31) / 32;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nblk; ++b) {
        double x[32], y[32];
        for (int d = 0; d < D; ++d) {
            for (int t = 0; t < 32; ++t) {
                const int64_t j = b * 32 + t;
                x[t] = (j < S) ? (double)oracle_bf16_to_f32(v[j * D + d]) : 0.0;
            }
            const int sc = block_e4m3_as_seen(x, 32, 0, y);
            if (scales) scales[b * D + d] = (uint8_t)sc;
            for (int t = 0; t < 32; ++t) {
                const int64_t j = b * 32 + t;
                if (j < n && j < S) seen[j * D + d] = y[t];
            }
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------ */
/* Alternative roundings (for the parity tests; no part of the method)                          */
/* ------------------------------------------------------------------------------------------ */
/* Rounding a probability for the second product is a decision taken on a floating-point value.
 * An implementation that forms the scores in binary32 sees a p that differs from the double p by
 * a few units in the last place of the score, and where the double p lies that close to the
 * midpoint of two representable numbers it legitimately picks the other one.  A parity test that
 * meets such a row asks for the row again with named decisions taken the other way (row_alts),
 * and compares the implementation with THAT result at the plain bar; which decisions are open to
 * this is decided by oracle_dma_attn_row_candidates() further down, not here.
 *   ORACLE_ALT_NEIGHBOUR   the probability of that key takes the other of its two neighbours
 *   ORACLE_ALT_SCALE_UP / _DOWN   (MX-format P V) the 32-key block of that key takes a shared
 *                          scale one binade coarser / finer than the rule gives */
#define ORACLE_ALT_NEIGHBOUR 1
#define ORACLE_ALT_SCALE_UP 2
#define ORACLE_ALT_SCALE_DOWN 3
typedef struct { int64_t n; const int64_t *key; const int32_t *kind; } row_alts;

static int alt_neighbour(const row_alts *alt, int64_t j)
{
    for (int64_t f = 0; alt && f < alt->n; ++f)
        if (alt->key[f] == j && alt->kind[f] == ORACLE_ALT_NEIGHBOUR) return 1;
    return 0;
}
static int alt_scale_shift(const row_alts *alt, int64_t j0, int n)      /* for the block of keys j0 .. j0+n-1 */
{
    for (int64_t f = 0; alt && f < alt->n; ++f)
        if (alt->key[f] >= j0 && alt->key[f] < j0 + n && alt->kind[f] != ORACLE_ALT_NEIGHBOUR)
            return alt->kind[f] == ORACLE_ALT_SCALE_UP ? 1 : -1;
    return 0;
}
/* rounded = p rounded to a grid of spacing 2^quantum around p: the grid point on the other side of p. */
static double other_grid_point(double p, double rounded, int quantum)
{
    const double lower = ldexp(floor(ldexp(p, -quantum)), quantum);
    if (lower == p) return rounded;                                      /* p is a grid point: nothing to decide */
    return (rounded == lower) ? lower + ldexp(1.0, quantum) : lower;
}
static int bf16_quantum(double p)                                      /* spacing of bf16 numbers at p > 0 is 2^this */
{
    int ex;
    (void)frexp(p, &ex);
    return (ex - 1) - 7 < -133 ? -133 : (ex - 1) - 7;
}
static int e4m3_quantum(double y)                                      /* spacing of E4M3 numbers at y > 0 is 2^this */
{
    int ex;
    (void)frexp(y, &ex);
    return (ex - 1) - 3 < -9 ? -9 : (ex - 1) - 3;
}
/* p seen as `seen` through an E4M3 block with scale byte sc: the other neighbour (none if p is clamped). */
static double e4m3_other_neighbour(double p, int sc, double seen)
{
    const double y = ldexp(p, 127 - sc);
    if (!(y > 0.0) || y >= 448.0) return seen;
    return ldexp(other_grid_point(y, ldexp(seen, 127 - sc), e4m3_quantum(y)), sc - 127);
}

/* What a parity test may ask to see of a row besides its output: per key j the score s_j (masked
 * keys: -inf) and the running maximum m' its tile ended with; the final m and l. */
typedef struct { double *s, *m; double m_final, l_final; } row_trace;

/* ------------------------------------------------------------------------------------------ */
/* Diagonal-tiled attention for a list of query rows (Alg. 1 + Sec. 3.2)                       */
/* ------------------------------------------------------------------------------------------ */

/* Output of one query row.  kseen_lo / kseen_hi: keys of this kv head as seen by the low / high
 * format, [S, D] doubles.  v: [S, D] bf16 of this kv head.
 *
 * Steps, in the paper's order, for the query tile it = i / tile:
 *   running state m = -inf, l = 1, O = 0                                   (Alg. 1 line 1)
 *   key tiles jt = 0 .. it ascending; Phase 1 = tiles before the window in the low format,
 *   Phase 2 = the last `band` tiles up to and including the diagonal one in the high format.
 *   Reading: the loop bounds are half open and n_Q*B_M means the END of the query tile, so a
 *   window of T = band * B_N tokens is exactly the last `band` key tiles ("only the last T
 *   tokens", Sec. 4.1).
 *   score s_j = q~ . k_j in that tile's format (Alg. 1 lines 3 and 7; base-2 scaling folded
 *   into q~, Alg. 2 Step 1); keys after the query are set to -inf (lines 8-9).
 *   Reading: -inf is selected where the mask holds (the printed S - inf*Delta would give NaN
 *   elsewhere), and the mask applies to the diagonal tile whatever its format.
 *   OnlineSoftmax (Sec. 3.2): m' = max(m, max_j s_j); alpha = 2^(m-m'); p_j = 2^(s_j - m');
 *   l = alpha*l + sum_j p_j;  O = alpha*O + sum_j p^_j * v_j;  finally O / l (line 12).
 *   Reading: p^_j = p_j rounded to bf16 when p_round = 1 (l sums the unrounded p_j).
 *   p_round = 2 (MX-format P V, beyond the paper): within the key tile, each block of 32 consecutive
 *   keys of the row's p_j (masked keys count as 0) is quantized to MXFP8-E4M3 as described above, V is
 *   taken as oracle_values_as_seen_mxfp8 gives it, and O accumulates the products of the two decoded
 *   values; l still sums the unrounded p_j.
 */
/* Extensions beyond Alg. 1 (both change only which key tiles are visited and in which format):
 *   sink  : the first `sink` key tiles are high precision for every query tile (Sec. 5.3, table
 *           of diagonal and sink windows).
 *   causal == 0 : every key tile is visited, nothing is masked, and the window is the tiles with
 *           |jt - it| < band (Sec. 4.1, "Compatibility with Non-Causal Attention").
 *   per_token : queries and keys go through Alg. 2 Step 2 (row divided by S_q = rowmax / 2688 before
 *           quantization, the decoded row multiplied by S_q again), the "Per-Token" granularity of
 *           Sec. 5.3; the scores are then S_q[i] * S_q[j] * (q^ . k^).  per_token = 2 / 3: the same with
 *           the maximum taken over the row's tile of its head ("Per-Block") / over the whole of Q
 *           resp. K ("Per-Tensor") instead of the row (oracle_group_amax).
 *   Reading: the printed tile ranges of the non-causal case mix index bases and the paper gives
 *   no loop for the sink window; it argues that any order that covers every tile once is valid.
 *   Here every variant visits the key tiles in ascending order, each in the format the rule
 *   above gives it; for causal attention without a sink this is exactly Phase 1 then Phase 2. */
/* alt / trace: NULL except when a parity test asks (see row_alts, row_trace above). */
static void attn_one_row(const uint16_t *qrow, const double *kseen_lo, const double *kseen_hi,
                         const uint16_t *v, const double *vseen, int64_t i, int64_t S, int D, int tile, int band, int sink,
                         int causal, int per_token, float q_amax, int hi_fmt, int lo_fmt, int p_round, float *out,
                         const row_alts *alt, row_trace *trace)
{
    double q_lo[512], q_hi[512], O[512];
    double *s = (double *)malloc(sizeof(double) * (size_t)tile * 3);
    double *pt = s + tile, *ph_t = s + 2 * tile;          /* p and its rounded image for the keys of a tile */
    row_as_seen(qrow, D, lo_fmt, 1, per_token, q_amax, q_lo);
    row_as_seen(qrow, D, hi_fmt, 1, per_token, q_amax, q_hi);
    const double c = 1.4426950408889634074 / sqrt((double)D);
    const double sc_lo = (lo_fmt == ORACLE_FMT_BF16) ? c : 1.0;   /* bf16 rows are not pre-scaled */
    const double sc_hi = (hi_fmt == ORACLE_FMT_BF16) ? c : 1.0;

    double m = -INFINITY, l = 1.0;
    for (int d = 0; d < D; ++d) O[d] = 0.0;

    const int64_t it = i / tile;
    const int64_t n_tiles = causal ? it + 1 : (S + tile - 1) / tile;   /* the last tile may be partial: keys >= S do not exist */
    for (int64_t jt = 0; jt < n_tiles; ++jt) {
        const int64_t dist = (it >= jt) ? it - jt : jt - it;
        const int use_hi = dist < (int64_t)band || jt < (int64_t)sink;
        const double *qq = use_hi ? q_hi : q_lo;
        const double *kk = use_hi ? kseen_hi : kseen_lo;
        const double sc = use_hi ? sc_hi : sc_lo;
        double tmax = -INFINITY;
        for (int t = 0; t < tile; ++t) {
            int64_t j = jt * tile + t;
            double acc;
            if ((causal && j > i) || j >= S) {
                acc = -INFINITY;
            } else {
                acc = 0.0;
                const double *kr = kk + j * D;
                for (int d = 0; d < D; ++d) acc += qq[d] * kr[d];
                acc *= sc;
            }
            s[t] = acc;
            if (acc > tmax) tmax = acc;
        }
        const double mnew = (tmax > m) ? tmax : m;
        const double alpha = exp2(m - mnew);
        double psum = 0.0;
        for (int d = 0; d < D; ++d) O[d] *= alpha;
        for (int t = 0; t < tile; ++t) {
            int64_t j = jt * tile + t;
            pt[t] = ((causal && j > i) || j >= S) ? 0.0 : exp2(s[t] - mnew);   /* 2^(-inf) = 0 */
            psum += pt[t];
            if (trace && j < S) { trace->s[j] = s[t]; trace->m[j] = mnew; }
        }
        if (p_round == 2) {
            /* MX-format P V: blocks of 32 keys of the tile */
            for (int t0 = 0; t0 < tile; t0 += 32) {
                const int n = (tile - t0 < 32) ? tile - t0 : 32;
                const int bsc = block_e4m3_as_seen(pt + t0, n, alt_scale_shift(alt, jt * tile + t0, n), ph_t + t0);
                for (int t = t0; alt && t < t0 + n; ++t)
                    if (alt_neighbour(alt, jt * tile + t)) ph_t[t] = e4m3_other_neighbour(pt[t], bsc, ph_t[t]);
            }
            for (int t = 0; t < tile; ++t) {
                const int64_t j = jt * tile + t;
                if (!(pt[t] > 0.0)) continue;
                const double *vr = vseen + j * D;
                for (int d = 0; d < D; ++d) O[d] += ph_t[t] * vr[d];
            }
        } else {
            for (int t = 0; t < tile; ++t) {
                int64_t j = jt * tile + t;
                if ((causal && j > i) || j >= S) continue; /* p = 2^(-inf) = 0 */
                double p = pt[t];
                double ph = p_round ? oracle_round_to_bf16(p) : p;
                if (p_round && p > 0.0 && alt_neighbour(alt, j)) ph = other_grid_point(p, ph, bf16_quantum(p));
                const uint16_t *vr = v + j * D;
                for (int d = 0; d < D; ++d) O[d] += ph * (double)oracle_bf16_to_f32(vr[d]);
            }
        }
        l = alpha * l + psum;
        m = mnew;
    }
    for (int d = 0; d < D; ++d) out[d] = (float)(O[d] / l);
    if (trace) { trace->m_final = m; trace->l_final = l; }
    free(s);
}

/* Keys of one kv head as seen in a format, rows 0 .. n-1, [n, D] doubles. */
static double *keys_as_seen(const uint16_t *k, int64_t n, int D, int fmt, int per_token, const float *amax_in)
{
    double *out = (double *)malloc(sizeof(double) * (size_t)n * (size_t)D);
    if (!out) return NULL;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n; ++r) row_as_seen(k + r * D, D, fmt, 0, per_token, amax_in ? amax_in[r] : -1.0f, out + r * D);
    return out;
}

/* The keys (both formats) and, for the MX-format P V, the values of one kv head as the products see
 * them, rows 0 .. n-1; and the group maxima of a coarser Step-2 granularity. */
typedef struct { double *klo, *khi, *vseen; } head_view;
static void head_view_free(head_view *h)
{
    if (h->khi != h->klo) free(h->khi);
    free(h->klo);
    free(h->vseen);
    h->klo = h->khi = h->vseen = NULL;
}
/* imax: the last key any of the rows to come will look at. */
static int head_view_make(head_view *h, const uint16_t *kh, const uint16_t *vh, int64_t S, int D, int tile, int64_t imax,
                          int per_token, const float *kam, int hi_fmt, int lo_fmt, int p_round)
{
    h->vseen = NULL;
    h->klo = keys_as_seen(kh, imax + 1, D, lo_fmt, per_token, kam);
    h->khi = (hi_fmt == lo_fmt) ? h->klo : keys_as_seen(kh, imax + 1, D, hi_fmt, per_token, kam);
    if (!h->klo || !h->khi) { head_view_free(h); return ORACLE_ERR_MEM; }
    if (p_round == 2) {
        /* every key of the tiles visited (whole 32-key blocks), but none past the end of the sequence */
        int64_t nv = ((imax + tile) / tile) * tile;
        if (nv > S) nv = S;
        h->vseen = (double *)malloc(sizeof(double) * (size_t)nv * (size_t)D);
        if (!h->vseen || oracle_values_as_seen_mxfp8(vh, S, D, nv, h->vseen, NULL) != ORACLE_OK) { head_view_free(h); return ORACLE_ERR_MEM; }
    }
    return ORACLE_OK;
}
static int attn_args_ok(const void *q, const void *k, const void *v, int B, int Hq, int Hkv, int64_t S, int D, int tile,
                        int band, int sink, int per_token, int hi_fmt, int lo_fmt, int p_round)
{
    if (!q || !k || !v || sink < 0) return 0;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || S <= 0 || D <= 0 || D % 32 != 0 || D > 512) return 0;
    if (tile <= 0 || band < 0) return 0;
    if (p_round < 0 || p_round > 2 || (p_round == 2 && tile % 32 != 0)) return 0;
    /* per_token: 0 = no Step 2; 1 = per-token; 2 = per-block (the rows of one tile of one head); 3 = per-tensor */
    if (per_token < 0 || per_token > 3) return 0;
    for (int f = 0; f < 2; ++f) {
        int fm = f ? hi_fmt : lo_fmt;
        if (fm != ORACLE_FMT_BF16 && !fmt_is_mx(fm)) return 0;
    }
    return 1;
}
/* Group maxima of all of Q and K for the per-block / per-tensor granularities (NULL, NULL otherwise). */
static int group_maxima_make(const uint16_t *q, const uint16_t *k, int B, int Hq, int Hkv, int64_t S, int D, int tile,
                             int per_token, float **qamax, float **kamax)
{
    *qamax = *kamax = NULL;
    if (per_token < 2) return ORACLE_OK;
    *qamax = (float *)malloc(sizeof(float) * (size_t)B * Hq * S);
    *kamax = (float *)malloc(sizeof(float) * (size_t)B * Hkv * S);
    if (!*qamax || !*kamax || oracle_group_amax(q, (int64_t)B * Hq, S, D, 1, per_token, tile, *qamax) != ORACLE_OK ||
        oracle_group_amax(k, (int64_t)B * Hkv, S, D, 0, per_token, tile, *kamax) != ORACLE_OK) {
        free(*qamax); free(*kamax); *qamax = *kamax = NULL;
        return ORACLE_ERR_MEM;
    }
    return ORACLE_OK;
}

/*
 * q: [B, Hq, S, D] bf16; k, v: [B, Hkv, S, D] bf16 (contiguous, D innermost; q head h uses kv
 * head h / (Hq/Hkv)).  rows: n_rows triples (b, hq, i).  out: [n_rows, D] float, in the order
 * of `rows`.  tile = B_M = B_N; band = T / B_N (0: every tile low; >= S/tile: every tile high).
 * Rows should be grouped by (b, kv head) for speed; any order is correct.
 */
int oracle_dma_attn_rows_ex(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int Hq,
                            int Hkv, int64_t S, int D, int tile, int band, int sink, int causal,
                            int per_token, int hi_fmt, int lo_fmt, int p_round, const int64_t *rows,
                            int64_t n_rows, float *out)
{
    if (!out || (!rows && n_rows > 0)) return ORACLE_ERR_ARG;
    if (!attn_args_ok(q, k, v, B, Hq, Hkv, S, D, tile, band, sink, per_token, hi_fmt, lo_fmt, p_round)) return ORACLE_ERR_ARG;
    for (int64_t r = 0; r < n_rows; ++r) {
        if (rows[3 * r] < 0 || rows[3 * r] >= B || rows[3 * r + 1] < 0 || rows[3 * r + 1] >= Hq ||
            rows[3 * r + 2] < 0 || rows[3 * r + 2] >= S)
            return ORACLE_ERR_ARG;
    }
    const int group = Hq / Hkv;
    float *qamax, *kamax;
    if (group_maxima_make(q, k, B, Hq, Hkv, S, D, tile, per_token, &qamax, &kamax) != ORACLE_OK) return ORACLE_ERR_MEM;
    int64_t r0 = 0;
    while (r0 < n_rows) {
        /* maximal run of rows sharing (b, kv head) */
        const int64_t b = rows[3 * r0], hkv = rows[3 * r0 + 1] / group;
        int64_t r1 = r0, imax = 0;
        while (r1 < n_rows && rows[3 * r1] == b && rows[3 * r1 + 1] / group == hkv) {
            if (rows[3 * r1 + 2] > imax) imax = rows[3 * r1 + 2];
            ++r1;
        }
        if (!causal) imax = S - 1;
        const uint16_t *kh = k + ((int64_t)b * Hkv + hkv) * S * D;
        const uint16_t *vh = v + ((int64_t)b * Hkv + hkv) * S * D;
        const float *kam = kamax ? kamax + ((int64_t)b * Hkv + hkv) * S : NULL;
        head_view hv;
        if (head_view_make(&hv, kh, vh, S, D, tile, imax, per_token, kam, hi_fmt, lo_fmt, p_round) != ORACLE_OK) {
            free(qamax); free(kamax); return ORACLE_ERR_MEM;
        }
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t r = r0; r < r1; ++r) {
            const int64_t hq = rows[3 * r + 1], i = rows[3 * r + 2];
            const uint16_t *qrow = q + (((int64_t)b * Hq + hq) * S + i) * D;
            const float qam = qamax ? qamax[((int64_t)b * Hq + hq) * S + i] : -1.0f;
            attn_one_row(qrow, hv.klo, hv.khi, vh, hv.vseen, i, S, D, tile, band, sink, causal, per_token, qam, hi_fmt, lo_fmt, p_round,
                         out + r * D, NULL, NULL);
        }
        head_view_free(&hv);
        r0 = r1;
    }
    free(qamax);
    free(kamax);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------ */
/* Parity-test support: which rounding decisions of a row are open, and the row with some of     */
/* them taken the other way.  Test infrastructure; no part of the method.                        */
/* ------------------------------------------------------------------------------------------ */
/* Score noise allowed to an implementation with binary32 scores, in units of the score: the score
 * and the running maximum are binary32 numbers that went through a handful of roundings each
 * (accumulation from -m, the moves of the maximum), so the exponent s - m' carries an error of a few
 * units in the last place of max(|s|, |m'|): 2^-22 (|s| + |m'| + 1) is two to four such units.
 * (Measured: the decisions the MI355X kernel takes the other way need at most a quarter of it.) */
static double score_noise(double s, double m) { return ldexp(fabs(s) + fabs(m) + 1.0, -22); }

/* A growing list of open decisions: key, kind, share of the noise allowance used, move of out[0..D). */
typedef struct { int64_t n, cap; int D; int64_t *key; int32_t *kind; double *used, *move; int failed; } open_list;
static void open_list_add(open_list *L, int64_t key, int32_t kind, double used, const double *move)
{
    if (L->failed) return;
    if (L->n == L->cap) {
        const int64_t cap = L->cap ? 2 * L->cap : 64;
        int64_t *k2 = (int64_t *)realloc(L->key, sizeof(int64_t) * (size_t)cap);
        if (k2) L->key = k2;
        int32_t *n2 = (int32_t *)realloc(L->kind, sizeof(int32_t) * (size_t)cap);
        if (n2) L->kind = n2;
        double *u2 = (double *)realloc(L->used, sizeof(double) * (size_t)cap);
        if (u2) L->used = u2;
        double *m2 = (double *)realloc(L->move, sizeof(double) * (size_t)cap * (size_t)L->D);
        if (m2) L->move = m2;
        if (!k2 || !n2 || !u2 || !m2) { L->failed = 1; return; }
        L->cap = cap;
    }
    L->key[L->n] = key; L->kind[L->n] = kind; L->used[L->n] = used;
    memcpy(L->move + L->n * L->D, move, sizeof(double) * (size_t)L->D);
    ++L->n;
}
static double largest_abs(const double *x, int n)
{
    double big = 0.0;
    for (int t = 0; t < n; ++t)
        if (fabs(x[t]) > big) big = fabs(x[t]);
    return big;
}

/* The open decisions of one row, from its trace (scores tr->s, running maxima tr->m, final m and l).
 *   bf16 P (p_round = 1): p_j lies within score_noise * ln2 * p_j of the midpoint of its two bf16 neighbours;
 *   MX-format P V (p_round = 2): the same against the E4M3 grid of the block's scale (kind NEIGHBOUR); and the
 *   block's scale itself when the block maximum of s - m' lies within score_noise of an integer (one binade
 *   finer if it may fall below that integer: SCALE_DOWN; coarser if it may reach it: SCALE_UP), or, for the block
 *   that holds the row maximum (s - m' = 0 exactly), when another key of the row comes that close to the maximum.
 * The move of a decision is its first-order effect on out[]: (new weight - old weight) * value * 2^(m' - m_final) / l
 * (the row sum adds the unrounded p and does not change).  values[j*D + d]: what key j contributes per unit weight. */
static void list_open_decisions(const row_trace *tr, int64_t n_keys, int tile, int D, int p_round, const double *values,
                                double min_move, open_list *L)
{
    double *mv = (double *)malloc(sizeof(double) * (size_t)D);
    if (!mv) { L->failed = 1; return; }
    /* single probabilities */
    for (int64_t j = 0; j < n_keys; ++j) {
        if (!(tr->s[j] > -INFINITY)) continue;                       /* masked */
        const double mj = tr->m[j];
        const double p = exp2(tr->s[j] - mj);
        if (!(p > 0.0)) continue;
        double rounded, other, spacing;
        if (p_round == 2) {
            /* the E4M3 grid at the scale of the key's 32-key block (keys of one block share a key tile, hence m') */
            const int64_t j0 = (j / 32) * 32;
            double pblk[32], seen[32];
            for (int t = 0; t < 32; ++t)
                pblk[t] = (j0 + t < n_keys && tr->s[j0 + t] > -INFINITY) ? exp2(tr->s[j0 + t] - mj) : 0.0;
            const int bsc = block_e4m3_as_seen(pblk, 32, 0, seen);
            const double y = ldexp(p, 127 - bsc);
            if (y >= 448.0) continue;                                /* clamped either way */
            spacing = ldexp(1.0, e4m3_quantum(y) + bsc - 127);
            rounded = seen[j - j0];
            other = e4m3_other_neighbour(p, bsc, rounded);
        } else {
            spacing = ldexp(1.0, bf16_quantum(p));
            rounded = oracle_round_to_bf16(p);
            other = other_grid_point(p, rounded, bf16_quantum(p));
        }
        if (other == rounded) continue;                              /* p is a grid point: nothing to decide */
        const double r = p / spacing;
        const double to_midpoint = fabs(r - floor(r) - 0.5) * spacing;
        const double allowance = score_noise(tr->s[j], mj) * 0.6931471805599453 * p;
        if (to_midpoint > allowance) continue;
        const double carry = exp2(mj - tr->m_final) / tr->l_final;
        for (int d = 0; d < D; ++d) mv[d] = (other - rounded) * values[j * D + d] * carry;
        if (largest_abs(mv, D) >= min_move) open_list_add(L, j, ORACLE_ALT_NEIGHBOUR, to_midpoint / allowance, mv);
    }
    /* shared scales of the 32-key blocks of P (MX-format P V only) */
    for (int64_t j0 = 0; p_round == 2 && j0 < n_keys; j0 += 32) {
        const int nb = (int)((n_keys - j0 < 32) ? n_keys - j0 : 32);
        const double mblk = tr->m[j0];
        double xmax = -INFINITY, second = -INFINITY;
        for (int t = 0; t < nb; ++t)
            if (tr->s[j0 + t] - mblk > xmax) xmax = tr->s[j0 + t] - mblk;
        if (xmax == -INFINITY) continue;                             /* every key masked */
        /* the largest s - m' of the row outside this block among the keys seen up to this tile */
        const int64_t tile_end = ((j0 / tile) + 1) * (int64_t)tile < n_keys ? ((j0 / tile) + 1) * (int64_t)tile : n_keys;
        for (int64_t j = 0; j < tile_end; ++j)
            if ((j < j0 || j >= j0 + nb) && tr->s[j] - mblk > second) second = tr->s[j] - mblk;
        const double noise = score_noise(xmax + mblk, mblk);
        int shift = 0;
        double used = 0.0;
        if (xmax == 0.0) { if (second >= -noise) { shift = -1; used = -second / noise; } }
        else if (xmax - floor(xmax) <= noise) { shift = -1; used = (xmax - floor(xmax)) / noise; }
        else if (ceil(xmax) - xmax <= noise) { shift = 1; used = (ceil(xmax) - xmax) / noise; }
        if (shift == 0) continue;
        double pblk[32], seen0[32], seen1[32];
        for (int t = 0; t < 32; ++t) pblk[t] = (t < nb && tr->s[j0 + t] > -INFINITY) ? exp2(tr->s[j0 + t] - mblk) : 0.0;
        (void)block_e4m3_as_seen(pblk, 32, 0, seen0);
        (void)block_e4m3_as_seen(pblk, 32, shift, seen1);
        const double carry = exp2(mblk - tr->m_final) / tr->l_final;
        for (int d = 0; d < D; ++d) {
            double acc = 0.0;
            for (int t = 0; t < nb; ++t) acc += (seen1[t] - seen0[t]) * values[(j0 + t) * D + d];
            mv[d] = acc * carry;
        }
        if (largest_abs(mv, D) >= min_move)
            open_list_add(L, j0, shift > 0 ? ORACLE_ALT_SCALE_UP : ORACLE_ALT_SCALE_DOWN, used, mv);
    }
    free(mv);
}

/* One row (b, hq, i), everything else as oracle_dma_attn_rows_ex (the probabilities are rounded: p_round 1 or 2).
 * alt_key / alt_kind [n_alt]: decisions to take the other way (ORACLE_ALT_*); out [D] receives the row.
 * With cand_key non-NULL (then n_alt must be 0) the open decisions of the row as the method rounds it are listed too,
 * largest move first: cand_key / cand_kind / cand_margin [max_cand] (margin = share of the noise allowance the
 * decision uses: 0 on the midpoint, 1 only just open), cand_move [max_cand, D]; *n_cand = how many there are whose
 * move reaches min_move in some out[d] (all of them counted, the first max_cand listed). */
int oracle_dma_attn_row_alt(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int Hq, int Hkv, int64_t S,
                            int D, int tile, int band, int sink, int causal, int per_token, int hi_fmt, int lo_fmt,
                            int p_round, int64_t b, int64_t hq, int64_t i, const int64_t *alt_key,
                            const int32_t *alt_kind, int64_t n_alt, float *out, double min_move, int64_t max_cand,
                            int64_t *cand_key, int32_t *cand_kind, double *cand_move, double *cand_margin, int64_t *n_cand)
{
    if (!out || n_alt < 0 || (n_alt > 0 && (!alt_key || !alt_kind))) return ORACLE_ERR_ARG;
    if (!attn_args_ok(q, k, v, B, Hq, Hkv, S, D, tile, band, sink, per_token, hi_fmt, lo_fmt, p_round)) return ORACLE_ERR_ARG;
    if (b < 0 || b >= B || hq < 0 || hq >= Hq || i < 0 || i >= S) return ORACLE_ERR_ARG;
    const int want_cand = cand_key != NULL;
    if (want_cand && (!cand_kind || !cand_move || !cand_margin || !n_cand || max_cand < 0 || n_alt != 0 || p_round == 0)) return ORACLE_ERR_ARG;
    const int64_t hkv = hq / (Hq / Hkv);
    const int64_t imax = causal ? i : S - 1;
    const uint16_t *kh = k + ((int64_t)b * Hkv + hkv) * S * D;
    const uint16_t *vh = v + ((int64_t)b * Hkv + hkv) * S * D;
    float *qamax, *kamax;
    if (group_maxima_make(q, k, B, Hq, Hkv, S, D, tile, per_token, &qamax, &kamax) != ORACLE_OK) return ORACLE_ERR_MEM;
    head_view hv;
    if (head_view_make(&hv, kh, vh, S, D, tile, imax, per_token, kamax ? kamax + ((int64_t)b * Hkv + hkv) * S : NULL, hi_fmt,
                       lo_fmt, p_round) != ORACLE_OK) {
        free(qamax); free(kamax); return ORACLE_ERR_MEM;
    }
    const uint16_t *qrow = q + (((int64_t)b * Hq + hq) * S + i) * D;
    const float qam = qamax ? qamax[((int64_t)b * Hq + hq) * S + i] : -1.0f;
    const row_alts alt = { n_alt, alt_key, alt_kind };
    const int64_t n_keys = ((imax / tile) + 1) * tile < S ? ((imax / tile) + 1) * tile : S;   /* keys of the tiles visited */
    row_trace tr = { NULL, NULL, 0.0, 0.0 };
    double *values = NULL;
    int rc = ORACLE_OK;
    if (want_cand) {
        tr.s = (double *)malloc(sizeof(double) * (size_t)n_keys * 2);
        values = (p_round == 2) ? hv.vseen : (double *)malloc(sizeof(double) * (size_t)n_keys * (size_t)D);
        if (!tr.s || !values) rc = ORACLE_ERR_MEM;
        tr.m = tr.s + n_keys;
        if (rc == ORACLE_OK && p_round != 2)
            for (int64_t e = 0; e < n_keys * D; ++e) values[e] = (double)oracle_bf16_to_f32(vh[e]);
    }
    if (rc == ORACLE_OK)
        attn_one_row(qrow, hv.klo, hv.khi, vh, hv.vseen, i, S, D, tile, band, sink, causal, per_token, qam, hi_fmt, lo_fmt, p_round,
                     out, n_alt ? &alt : NULL, want_cand ? &tr : NULL);
    if (rc == ORACLE_OK && want_cand) {
        open_list L = { 0, 0, D, NULL, NULL, NULL, NULL, 0 };
        list_open_decisions(&tr, n_keys, tile, D, p_round, values, min_move, &L);
        if (L.failed) {
            rc = ORACLE_ERR_MEM;
        } else {
            *n_cand = L.n;
            for (int64_t a = 0; a < L.n && a < max_cand; ++a) {           /* selection of the largest moves, in order */
                int64_t best = -1;
                double bestv = -1.0;
                for (int64_t c2 = 0; c2 < L.n; ++c2) {
                    if (L.kind[c2] == 0) continue;                         /* taken */
                    const double big = largest_abs(L.move + c2 * D, D);
                    if (big > bestv) { bestv = big; best = c2; }
                }
                cand_key[a] = L.key[best]; cand_kind[a] = L.kind[best]; cand_margin[a] = L.used[best];
                memcpy(cand_move + a * D, L.move + best * D, sizeof(double) * (size_t)D);
                L.kind[best] = 0;
            }
        }
        free(L.key); free(L.kind); free(L.used); free(L.move);
    }
    if (values != hv.vseen) free(values);
    free(tr.s);
    head_view_free(&hv);
    free(qamax);
    free(kamax);
    return rc;
}

/* Alg. 1 as printed: causal, no sink window. */
int oracle_dma_attn_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int Hq,
                         int Hkv, int64_t S, int D, int tile, int band, int hi_fmt, int lo_fmt,
                         int p_round, const int64_t *rows, int64_t n_rows, float *out)
{
    return oracle_dma_attn_rows_ex(q, k, v, B, Hq, Hkv, S, D, tile, band, 0, 1, 0, hi_fmt, lo_fmt, p_round, rows,
                                   n_rows, out);
}

/* ------------------------------------------------------------------------------------------ */
/* Exact softmax attention of the unquantized inputs (Sec. 3.2, eq. 1), causal or not, for      */
/* reporting the method's own error.  Natural-base softmax of q.k/sqrt(D), two passes, double. */
/* ------------------------------------------------------------------------------------------ */
int oracle_ref_attn_rows_ex(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int Hq,
                            int Hkv, int64_t S, int D, int causal, const int64_t *rows, int64_t n_rows,
                            double *out)
{
    if (!q || !k || !v || !out || (!rows && n_rows > 0)) return ORACLE_ERR_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || S <= 0 || D <= 0) return ORACLE_ERR_ARG;
    for (int64_t r = 0; r < n_rows; ++r) {
        if (rows[3 * r] < 0 || rows[3 * r] >= B || rows[3 * r + 1] < 0 || rows[3 * r + 1] >= Hq ||
            rows[3 * r + 2] < 0 || rows[3 * r + 2] >= S)
            return ORACLE_ERR_ARG;
    }
    const int group = Hq / Hkv;
    const double inv = 1.0 / sqrt((double)D);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t b = rows[3 * r], hq = rows[3 * r + 1], i = rows[3 * r + 2];
        const uint16_t *qrow = q + ((b * Hq + hq) * S + i) * D;
        const uint16_t *kh = k + (b * Hkv + hq / group) * S * D;
        const uint16_t *vh = v + (b * Hkv + hq / group) * S * D;
        const int64_t jmax = causal ? i : S - 1;        /* last key this row attends to */
        double *s = (double *)malloc(sizeof(double) * (size_t)(jmax + 1));
        if (!s) { err = 1; continue; }
        double mx = -INFINITY;
        for (int64_t j = 0; j <= jmax; ++j) {
            double acc = 0.0;
            for (int d = 0; d < D; ++d)
                acc += (double)oracle_bf16_to_f32(qrow[d]) * (double)oracle_bf16_to_f32(kh[j * D + d]);
            s[j] = acc * inv;
            if (s[j] > mx) mx = s[j];
        }
        double den = 0.0;
        double *o = out + r * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int64_t j = 0; j <= jmax; ++j) {
            double p = exp(s[j] - mx);
            den += p;
            for (int d = 0; d < D; ++d) o[d] += p * (double)oracle_bf16_to_f32(vh[j * D + d]);
        }
        for (int d = 0; d < D; ++d) o[d] /= den;
        free(s);
    }
    return err ? ORACLE_ERR_MEM : ORACLE_OK;
}

int oracle_ref_attn_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int Hq,
                         int Hkv, int64_t S, int D, const int64_t *rows, int64_t n_rows, double *out)
{
    return oracle_ref_attn_rows_ex(q, k, v, B, Hq, Hkv, S, D, 1, rows, n_rows, out);
}

/* Number of OpenMP threads the loops above use (for reporting the CPU baseline). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
