/*
 * CPU oracle for the three serving operators of the Astra paper (arxiv 2509.07506, Table 1):
 *   Kernel 1  merge_attn_states_lse   V_out = (e^Sa Va + e^Sb Vb)/(e^Sa + e^Sb),  S_out = log(e^Sa + e^Sb)
 *   Kernel 2  fused_add_rmsnorm       y = (x+r) / sqrt(||x+r||^2 / D + eps) (.) w
 *   Kernel 3  silu_and_mul            out = SiLU(x) (.) g,  SiLU(z) = z / (1 + e^-z)
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, scalar implementation used only
 * by the test-suite, the smoke check and the benchmark's CPU-baseline leg to judge the HIP library.
 * It shares no code, header, table or helper with the HIP path and the product never calls it.
 *
 * Arithmetic: every operator is evaluated in IEEE binary32 with the operations in the order the
 * formula states, one rounding to the 16-bit storage type at the very end.  Compile without FMA
 * contraction and without fast-math (-ffp-contract=off) so that a*x + b*y is two products and one
 * sum, which makes the merge bit-exactly symmetric in its two inputs.
 *
 * Storage types: 0 = IEEE binary16 (fp16), 1 = bfloat16.  Widening to binary32 is exact.  Narrowing
 * is round-to-nearest-even, overflow goes to +-inf, NaN stays a quiet NaN, subnormals are kept.
 * The conversions are written out by hand below (bit manipulation only).
 *
 * Pins (see tests/test_oracle_*.py): conversions against numpy's float16 cast, against torch's
 * bfloat16 cast and against a brute-force nearest-neighbour search; rmsnorm against unit-RMS,
 * constant-row, power-of-two scale invariance, r = 0 textbook RMSNorm in float64; silu against
 * silu(0) = 0, silu(x) - silu(-x) = x, the tanh identity, asymptotes and the location of the
 * minimum; merge against brute-force softmax attention over the concatenated key sets, symmetry,
 * one-sided -inf, equal scores, shift invariance, convexity and associativity.
 *
 * Conventions the paper leaves open (each restated where it is used):
 *   - sum of squares is taken over the unrounded binary32 sum x+r;
 *   - input <- y and residual <- x+r (both in place);
 *   - the first half of a silu_and_mul input row is x (activated), the second half is g;
 *   - both scores -inf gives V_out = 0 and S_out = -inf (the listing in Fig. 2 guards the
 *     denominator with a tiny constant, which makes the weights 0 in this case; Table 1 has no
 *     such constant and for any finite score the constant vanishes in binary32).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

/* ------------------------------------------------------------------------------------------- */
/* bit casts                                                                                   */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* shift right by `sh` (1..31) with round-to-nearest, ties to even */
static uint32_t shr_rne(uint32_t v, unsigned sh)
{
    uint32_t q = v >> sh;
    uint32_t rem = v & ((1u << sh) - 1u);
    uint32_t half = 1u << (sh - 1);
    if (rem > half || (rem == half && (q & 1u))) q += 1u;
    return q;
}

/* ------------------------------------------------------------------------------------------- */
/* bfloat16: the upper 16 bits of a binary32                                                   */

float oracle_bf16_to_f32(uint16_t h) { return bits_f32((uint32_t)h << 16); }

uint16_t oracle_f32_to_bf16(float f)
{
    uint32_t u = f32_bits(f);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t mag = u & 0x7fffffffu;
    if (mag > 0x7f800000u) return (uint16_t)(sign | 0x7fc0u);          /* NaN -> quiet NaN */
    /* finite or inf: drop 16 bits with RNE; a carry out of the mantissa moves into the exponent
       and max-finite + half ulp carries into the inf pattern, which is the IEEE overflow rule */
    return (uint16_t)(sign | shr_rne(mag, 16));
}

/* ------------------------------------------------------------------------------------------- */
/* binary16: 1 sign, 5 exponent (bias 15), 10 mantissa bits                                    */

float oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu;
    uint32_t m = h & 0x3ffu;
    if (e == 0x1fu) return bits_f32(sign | 0x7f800000u | (m << 13));   /* inf / NaN */
    if (e != 0) return bits_f32(sign | ((e + 112u) << 23) | (m << 13)); /* normal: rebias 15->127 */
    /* zero or subnormal: value = m * 2^-24, exactly representable */
    {
        float v = (float)m * 5.9604644775390625e-08f; /* 2^-24 */
        return sign ? -v : v;
    }
}

uint16_t oracle_f32_to_f16(float f)
{
    uint32_t u = f32_bits(f);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t mag = u & 0x7fffffffu;
    uint32_t e = mag >> 23;
    if (mag > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);          /* NaN */
    if (mag >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);         /* >= 65520 rounds to inf */
    if (e >= 113u) {
        /* normal half: rebias the exponent (127 -> 15) and drop 13 mantissa bits with RNE;
           a mantissa carry correctly bumps the exponent */
        return (uint16_t)(sign | shr_rne(mag - (112u << 23), 13));
    }
    /* below 2^-14: result is an integer multiple q of 2^-24 with q = round(|f| * 2^24).
       |f| = M * 2^(e-150) with M the 24-bit significand, so q = M >> (126 - e). */
    if (e < 101u) return (uint16_t)sign;                               /* < 2^-26: rounds to 0 */
    {
        uint32_t M = (mag & 0x7fffffu) | 0x800000u;
        return (uint16_t)(sign | shr_rne(M, 126u - e));
    }
}

static float widen(uint16_t h, int dtype)
{
    return dtype == ORACLE_BF16 ? oracle_bf16_to_f32(h) : oracle_f16_to_f32(h);
}

static uint16_t narrow(float f, int dtype)
{
    return dtype == ORACLE_BF16 ? oracle_f32_to_bf16(f) : oracle_f32_to_f16(f);
}

/* array forms, used by the conversion pins */
void oracle_widen_array(const uint16_t* in, float* out, int64_t n, int dtype)
{
    for (int64_t i = 0; i < n; ++i) out[i] = widen(in[i], dtype);
}

void oracle_narrow_array(const float* in, uint16_t* out, int64_t n, int dtype)
{
    for (int64_t i = 0; i < n; ++i) out[i] = narrow(in[i], dtype);
}

/* ------------------------------------------------------------------------------------------- */
/* threads: rows are independent, so the only parallelism is an OpenMP loop over rows          */

static int g_threads = 1;

void oracle_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int oracle_get_threads(void)
{
#ifdef _OPENMP
    return g_threads;
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------- */
/* Kernel 2: fused_add_rmsnorm (Table 1, second row)                                           */

/* One row, all binary32.  s_j = x_j + r_j ; ms = (sum_j s_j^2) / H ; y_j = s_j / sqrt(ms + eps) * w_j.
   The sum runs left to right. */
static void rmsnorm_row_f32(const float* x, const float* r, const float* w, int64_t H, float eps,
                            float* s, float* y)
{
    float sumsq = 0.0f;
    for (int64_t j = 0; j < H; ++j) {
        s[j] = x[j] + r[j];
        sumsq += s[j] * s[j];
    }
    {
        float ms = sumsq / (float)H;
        float inv = 1.0f / sqrtf(ms + eps);
        for (int64_t j = 0; j < H; ++j) y[j] = (s[j] * inv) * w[j];
    }
}

/* All-binary32 form (no storage rounding): s_out = x + r, y_out = normalised and weighted row. */
void oracle_fused_add_rmsnorm_f32(const float* x, const float* r, const float* w, int64_t T, int64_t H,
                                  float eps, float* s_out, float* y_out)
{
    for (int64_t t = 0; t < T; ++t)
        rmsnorm_row_f32(x + t * H, r + t * H, w, H, eps, s_out + t * H, y_out + t * H);
}

/* Storage form: input[T,H], residual[T,H], weight[H] hold 16-bit patterns of `dtype`.
   residual <- RNE(x + r) (bit-defined: one binary32 add, one rounding); input <- RNE(y).
   The normalisation uses the unrounded binary32 sum, not the stored residual. */
void oracle_fused_add_rmsnorm(uint16_t* input, uint16_t* residual, const uint16_t* weight, int64_t T,
                              int64_t H, int dtype, float eps)
{
    float* wf = (float*)malloc(sizeof(float) * (size_t)(H > 0 ? H : 1));
    for (int64_t j = 0; j < H; ++j) wf[j] = widen(weight[j], dtype);
#pragma omp parallel num_threads(g_threads)
    {
        float* buf = (float*)malloc(sizeof(float) * 4 * (size_t)(H > 0 ? H : 1));
        float *xf = buf, *rf = buf + H, *s = buf + 2 * H, *y = buf + 3 * H;
#pragma omp for schedule(static)
        for (int64_t t = 0; t < T; ++t) {
            uint16_t* xi = input + t * H;
            uint16_t* ri = residual + t * H;
            for (int64_t j = 0; j < H; ++j) {
                xf[j] = widen(xi[j], dtype);
                rf[j] = widen(ri[j], dtype);
            }
            rmsnorm_row_f32(xf, rf, wf, H, eps, s, y);
            for (int64_t j = 0; j < H; ++j) {
                ri[j] = narrow(s[j], dtype);
                xi[j] = narrow(y[j], dtype);
            }
        }
        free(buf);
    }
    free(wf);
}

/* ------------------------------------------------------------------------------------------- */
/* Kernel 3: silu_and_mul (Table 1, third row; the plain form of Fig. 5a)                      */

float oracle_silu_f32(float z) { return z / (1.0f + expf(-z)); }

/* in[T, 2d]: columns [0,d) are x (activated), columns [d,2d) are g.  out[T,d] = RNE(silu(x) * g). */
void oracle_silu_and_mul(uint16_t* out, const uint16_t* in, int64_t T, int64_t d, int dtype)
{
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t t = 0; t < T; ++t) {
        const uint16_t* row = in + t * 2 * d;
        for (int64_t j = 0; j < d; ++j) {
            float x = widen(row[j], dtype);
            float g = widen(row[d + j], dtype);
            out[t * d + j] = narrow(oracle_silu_f32(x) * g, dtype);
        }
    }
}

/* All-binary32 form. */
void oracle_silu_and_mul_f32(float* out, const float* in, int64_t T, int64_t d)
{
    for (int64_t t = 0; t < T; ++t)
        for (int64_t j = 0; j < d; ++j) out[t * d + j] = oracle_silu_f32(in[t * 2 * d + j]) * in[t * 2 * d + d + j];
}

/* ------------------------------------------------------------------------------------------- */
/* Kernel 1: merge_attn_states_lse (Table 1, first row)                                        */

/* Mixing weights for one (token, head).  Dividing numerator and denominator of Table 1's formula
   by e^m, m = max(Sa, Sb), gives a = e^(Sa-m) / (e^(Sa-m) + e^(Sb-m)), likewise b, and
   S_out = m + log(e^(Sa-m) + e^(Sb-m)); the larger exponential is exactly 1, nothing overflows.
   Both scores -inf (two empty partitions): a = b = 0 and S_out = -inf. */
void oracle_merge_weights_f32(float sa, float sb, float* a, float* b, float* s_out)
{
    float m = fmaxf(sa, sb);
    if (m == -INFINITY) {
        *a = 0.0f;
        *b = 0.0f;
        *s_out = -INFINITY;
        return;
    }
    {
        float wa = expf(sa - m);
        float wb = expf(sb - m);
        float den = wa + wb;
        *a = wa / den;
        *b = wb / den;
        *s_out = m + logf(den);
    }
}

/* One element of the blend a * va + b * vb (two products and one sum).  A term whose weight is exactly zero is
   left out, its value is not looked at: an empty partition (score -inf) stands for attention over no keys, whose
   value vector is undefined, and Table 1's weighted mean over the union of the key sets does not depend on it.
   So one empty side returns the other side's term alone, whatever the empty side's buffer holds. */
static float blend2(float a, float va, float b, float vb)
{
    if (a == 0.0f && b == 0.0f) return 0.0f;
    if (a == 0.0f) return b * vb;
    if (b == 0.0f) return a * va;
    {
        float pa = a * va;
        float pb = b * vb;
        return pa + pb;
    }
}

/* v_a, v_b, v_out: [T, NH, D] 16-bit patterns of `dtype`; lse_a, lse_b, lse_out: [T, NH] binary32.
   v_out = RNE(a * v_a + b * v_b), zero-weight terms left out (blend2). */
void oracle_merge_attn_states_lse(uint16_t* v_out, float* lse_out, const uint16_t* v_a, const float* lse_a,
                                  const uint16_t* v_b, const float* lse_b, int64_t T, int64_t NH, int64_t D,
                                  int dtype)
{
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t p = 0; p < T * NH; ++p) {
        float a, b, s;
        oracle_merge_weights_f32(lse_a[p], lse_b[p], &a, &b, &s);
        lse_out[p] = s;
        for (int64_t k = 0; k < D; ++k)
            v_out[p * D + k] = narrow(blend2(a, widen(v_a[p * D + k], dtype), b, widen(v_b[p * D + k], dtype)), dtype);
    }
}

/* K-way merge: the K-term form of Table 1's Kernel 1,
     V_out = sum_k e^(S_k) V_k / sum_k e^(S_k),   S_out = log sum_k e^(S_k),
   evaluated with m = max_k S_k subtracted from every score.  The paper defines only K = 2; this is the
   same expression with more terms (merging is associative, so it equals any chain of two-way merges up
   to rounding).  v_parts: [K, P, D] patterns (P = T*NH pairs), lse_parts: [K, P] binary32.
   Terms are accumulated in the order k = 0, 1, ..., K-1; a term whose weight is exactly zero is left out, as in
   blend2.  All scores -inf: V_out = 0, S_out = -inf. */
void oracle_merge_attn_states_lse_kway(uint16_t* v_out, float* lse_out, const uint16_t* v_parts,
                                       const float* lse_parts, int64_t K, int64_t P, int64_t D, int dtype)
{
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t p = 0; p < P; ++p) {
        float m = -INFINITY;
        for (int64_t k = 0; k < K; ++k) m = fmaxf(m, lse_parts[k * P + p]);
        if (m == -INFINITY) {
            lse_out[p] = -INFINITY;
            for (int64_t j = 0; j < D; ++j) v_out[p * D + j] = narrow(0.0f, dtype);
            continue;
        }
        float den = 0.0f;
        for (int64_t k = 0; k < K; ++k) den += expf(lse_parts[k * P + p] - m);
        lse_out[p] = m + logf(den);
        for (int64_t j = 0; j < D; ++j) {
            float acc = 0.0f;
            for (int64_t k = 0; k < K; ++k) {
                float a = expf(lse_parts[k * P + p] - m) / den;
                if (a != 0.0f) acc += a * widen(v_parts[(k * P + p) * D + j], dtype);
            }
            v_out[p * D + j] = narrow(acc, dtype);
        }
    }
}

/* All-binary32 form of the K-way merge: the same three passes (maximum, denominator, weighted sum in the order
   k = 0 .. K-1, zero-weight terms left out) on float values; v_parts [K, P, D], lse_parts [K, P]. */
void oracle_merge_attn_states_lse_kway_f32(float* v_out, float* lse_out, const float* v_parts, const float* lse_parts,
                                           int64_t K, int64_t P, int64_t D)
{
    for (int64_t p = 0; p < P; ++p) {
        float top = -INFINITY;
        for (int64_t k = 0; k < K; ++k) top = fmaxf(top, lse_parts[k * P + p]);
        if (top == -INFINITY) { /* every partition empty */
            lse_out[p] = -INFINITY;
            for (int64_t j = 0; j < D; ++j) v_out[p * D + j] = 0.0f;
            continue;
        }
        float total = 0.0f;
        for (int64_t k = 0; k < K; ++k) total += expf(lse_parts[k * P + p] - top);
        lse_out[p] = top + logf(total);
        for (int64_t j = 0; j < D; ++j) {
            float sum = 0.0f;
            for (int64_t k = 0; k < K; ++k) {
                float wgt = expf(lse_parts[k * P + p] - top) / total;
                if (wgt != 0.0f) sum += wgt * v_parts[(k * P + p) * D + j];
            }
            v_out[p * D + j] = sum;
        }
    }
}

/* All-binary32 form. */
void oracle_merge_attn_states_lse_f32(float* v_out, float* lse_out, const float* v_a, const float* lse_a,
                                      const float* v_b, const float* lse_b, int64_t T, int64_t NH, int64_t D)
{
    for (int64_t p = 0; p < T * NH; ++p) {
        float a, b, s;
        oracle_merge_weights_f32(lse_a[p], lse_b[p], &a, &b, &s);
        lse_out[p] = s;
        for (int64_t k = 0; k < D; ++k) v_out[p * D + k] = blend2(a, v_a[p * D + k], b, v_b[p * D + k]);
    }
}
