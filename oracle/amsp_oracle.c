/*
 * CPU oracle for one rank's model-state step on its flat shard of P/G/OS.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, scalar, double precision.  It shares no
 * code with the HIP library and is never called by it; only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may use it.
 *
 * What it computes is a definition, not an approximation, so each function is that
 * definition written out, one loop, no blocking or reordering:
 *
 *   shard range   a flat buffer of Phi elements split evenly over s ranks (Section IV-B,
 *                 sharding factors; Section IV-C.2, intra-tensor "even split").
 *   reduce        G[i] = sum_j g_j[i]: what a rank holds after gradient synchronisation
 *                 (Section II-C ZeRO-2/3; Section IV-C.1 ReduceScatter; Section IV-C.2
 *                 AllReduce then select).  Sum, not mean.
 *   sqnorm/clip   S = sum_i G[i]^2, scale = min(1, c / (sqrt(S) + clip_eps)).  The paper
 *                 does not mention clipping; this is the usual global-L2 rule.
 *   AdamW         the update "each GPU applies to Phi/s_os parameters based on the
 *                 optimizer states" (Section IV-C.2) with Adam under mixed precision
 *                 (Section II-C: 12 bytes of fp32 master, m, v per parameter):
 *                     g' = scale G
 *                     m' = b1 m + (1-b1) g'
 *                     v' = b2 v + (1-b2) g'^2
 *                     p' = p - lr ( (m'/(1-b1^t)) / (sqrt(v'/(1-b2^t)) + eps) + wd p )
 *   cast          fp32 -> bf16, round to nearest even: the 2-byte parameter that the
 *                 AllGather/Broadcast of Section IV-C.2 ships (BF16 per Section VI).
 *
 * Hyper-parameters arrive as the fp32 values the library receives and are widened, so
 * both sides use identical constants.  All state inputs are the fp32 buffers widened.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static double bf16_value(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Rank r of s gets Phi/s elements; the first Phi%s ranks get one more.  Contiguous. */
void amsp_oracle_shard_range(uint64_t total, uint32_t s, uint32_t r, uint64_t *begin, uint64_t *end) {
    uint64_t base = total / s, rem = total % s;
    uint64_t extra_before = r < rem ? r : rem;
    *begin = (uint64_t)r * base + extra_before;
    *end = *begin + base + (r < rem ? 1u : 0u);
}

/* G[i] = sum over the k partial buffers, j = 0..k-1.  Exact in double for k <= 32
 * (each bf16 carries 8 significant bits) unless exponents spread over > 40 bits. */
void amsp_oracle_reduce(const uint16_t *const *partials, uint32_t k, uint64_t n, double *G) {
    for (uint64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (uint32_t j = 0; j < k; ++j) s += bf16_value(partials[j][i]);
        G[i] = s;
    }
}

/* Sum of squares; long double keeps the accumulated error far below the 1e-5 budget
 * at billions of elements. */
double amsp_oracle_sqnorm(const double *G, uint64_t n) {
    long double s = 0.0L;
    for (uint64_t i = 0; i < n; ++i) s += (long double)G[i] * (long double)G[i];
    return (double)s;
}

/* max_norm <= 0 switches clipping off. */
double amsp_oracle_clip_scale(double total_sqnorm, double max_norm, double clip_eps) {
    if (!(max_norm > 0.0)) return 1.0;
    double c = max_norm / (sqrt(total_sqnorm) + clip_eps);
    return c < 1.0 ? c : 1.0;
}

/* One AdamW step on n elements; t >= 1 is the index of the update being applied.
 * Results in double; the caller rounds to fp32 when it compares. */
void amsp_oracle_adamw(const double *G, double scale, const float *p, const float *m, const float *v,
                       uint64_t n, float lr_f, float beta1_f, float beta2_f, float eps_f, float wd_f,
                       uint32_t t, double *p_out, double *m_out, double *v_out) {
    const double lr = lr_f, b1 = beta1_f, b2 = beta2_f, eps = eps_f, wd = wd_f;
    const double bc1 = 1.0 - pow(b1, (double)t);
    const double bc2 = 1.0 - pow(b2, (double)t);
    for (uint64_t i = 0; i < n; ++i) {
        double g = scale * G[i];
        double m1 = b1 * (double)m[i] + (1.0 - b1) * g;
        double v1 = b2 * (double)v[i] + (1.0 - b2) * g * g;
        double mhat = m1 / bc1;
        double vhat = v1 / bc2;
        double pi = (double)p[i];
        p_out[i] = pi - lr * (mhat / (sqrt(vhat) + eps) + wd * pi);
        m_out[i] = m1;
        v_out[i] = v1;
    }
}

/* fp32 -> bf16 round-to-nearest-even on the bit pattern.  NaN -> quiet NaN with the
 * sign kept; +-Inf kept; finite overflow rounds to +-Inf; subnormals are rounded like
 * any other value (no flush). */
uint16_t amsp_oracle_bf16_rne(float x) {
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)(((u >> 16) & 0x8000u) | 0x7FC0u);
    uint32_t keep_lsb = (u >> 16) & 1u;
    u += 0x7FFFu + keep_lsb;
    return (uint16_t)(u >> 16);
}

void amsp_oracle_cast(const float *p, uint64_t n, uint16_t *out) {
    for (uint64_t i = 0; i < n; ++i) out[i] = amsp_oracle_bf16_rne(p[i]);
}

/* double -> fp32 (RNE, the C conversion) -> bf16: the shipped parameter for a double p'. */
void amsp_oracle_round_f32(const double *x, uint64_t n, float *out) {
    for (uint64_t i = 0; i < n; ++i) out[i] = (float)x[i];
}

/* ---------------------------------------------------------------------------------------------
 * FP8 payload with per-tensor scaling factors: the reason Section IV-C.2 gives for adopting
 * inter-tensor shards (each rank owns whole tensors, so one scale per tensor travels with them).
 * The paper fixes no format; taken here: OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa
 * bits, subnormals, no infinities, largest finite 448, NaN = S.1111.111), round to nearest even,
 * values beyond the largest finite SATURATE to +-448, and
 *     scale = 448 / amax(|tensor|)   (1 when amax is 0 or not finite),   code = e4m3(p * scale),
 * with amax, scale and the product taken in fp32, because they decide an integer code.
 */
float amsp_oracle_e4m3_decode(uint8_t c) {
    int sign = c >> 7, e = (c >> 3) & 0xF, m = c & 7;
    float v;
    if (e == 0xF && m == 7) v = NAN;
    else if (e == 0) v = ldexpf((float)m, -9);                 /* subnormal: m * 2^-9 */
    else v = ldexpf(1.0f + (float)m / 8.0f, e - 7);
    return sign ? -v : v;
}

uint8_t amsp_oracle_e4m3_encode(float x) {
    uint8_t sign = signbit(x) ? 0x80 : 0x00;
    if (isnan(x)) return sign | 0x7F;
    double a = fabs((double)x);
    if (a >= 464.0) return sign | 0x7E;                        /* 464 is the midpoint above 448: tie goes to even = 448 */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                                        /* a = f * 2^e, f in [0.5, 1) */
    e -= 1;                                                    /* a in [2^e, 2^(e+1)) */
    if (e < -6) e = -6;                                        /* subnormal range shares the spacing of 2^-6 */
    double q = ldexp(1.0, e - 3);                              /* grid spacing */
    double r = nearbyint(a / q);                               /* exact quotient, ties to even */
    if (r >= 16.0) { r = 8.0; e += 1; }
    if (r < 8.0) return sign | (uint8_t)r;                     /* subnormal codes 0..7 */
    return sign | (uint8_t)(((e + 7) << 3) | ((int)r - 8));
}

float amsp_oracle_absmax(const float *p, uint64_t n) {
    float a = 0.0f;
    for (uint64_t i = 0; i < n; ++i) {
        float v = fabsf(p[i]);
        if (v > a || isnan(v)) a = v;                          /* a NaN anywhere makes the result NaN */
        if (isnan(a)) break;
    }
    return a;
}

float amsp_oracle_fp8_scale(float amax) {
    if (!(amax > 0.0f) || !isfinite(amax)) return 1.0f;
    return 448.0f / amax;
}

void amsp_oracle_cast_fp8(const float *p, uint64_t n, float scale, uint8_t *out) {
    for (uint64_t i = 0; i < n; ++i) {
        volatile float x = p[i] * scale;                       /* one fp32 multiply, rounded to fp32 */
        out[i] = amsp_oracle_e4m3_encode(x);
    }
}
