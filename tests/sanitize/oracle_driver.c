/* Runs every function of the C oracle on seeded inputs at ragged sizes and prints one checksum per
 * call.  Built twice by tests/test_sanitizers_cpu.py, plain and with -fsanitize=address,undefined: both
 * builds must print the same lines, and the instrumented one must report nothing. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void amsp_oracle_shard_range(uint64_t total, uint32_t s, uint32_t r, uint64_t *begin, uint64_t *end);
void amsp_oracle_reduce(const uint16_t *const *partials, uint32_t k, uint64_t n, double *G);
double amsp_oracle_sqnorm(const double *G, uint64_t n);
double amsp_oracle_clip_scale(double total_sqnorm, double max_norm, double clip_eps);
void amsp_oracle_adamw(const double *G, double scale, const float *p, const float *m, const float *v,
                       uint64_t n, float lr, float beta1, float beta2, float eps, float wd, uint32_t step,
                       double *p_out, double *m_out, double *v_out);
uint16_t amsp_oracle_bf16_rne(float x);
void amsp_oracle_cast(const float *p, uint64_t n, uint16_t *out);
void amsp_oracle_round_f32(const double *x, uint64_t n, float *out);
float amsp_oracle_e4m3_decode(uint8_t c);
uint8_t amsp_oracle_e4m3_encode(float x);
float amsp_oracle_absmax(const float *p, uint64_t n);
float amsp_oracle_fp8_scale(float amax);
void amsp_oracle_cast_fp8(const float *p, uint64_t n, float scale, uint8_t *out);

static uint64_t state = 0x2311002570000003ull;
static uint64_t rnd(void) {
    uint64_t z = (state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static uint64_t fnv(const void *data, size_t bytes, uint64_t h) {
    const unsigned char *b = (const unsigned char *)data;
    for (size_t i = 0; i < bytes; ++i) h = (h ^ b[i]) * 0x100000001B3ull;
    return h;
}
/* exactly n elements each (malloc(0) is replaced by a one-byte block nobody may read past) */
static void *room(size_t bytes) {
    void *p = malloc(bytes ? bytes : 1);
    if (!p) exit(3);
    return p;
}
static float some_float(int wild) {
    uint32_t u = (uint32_t)rnd();
    if (!wild) u = (u & 0x807FFFFFu) | ((uint32_t)(100 + rnd() % 40) << 23);   /* 2^-27 .. 2^12 */
    float f;
    memcpy(&f, &u, 4);
    return f;
}

int main(void) {
    const uint64_t sizes[] = {0, 1, 2, 3, 7, 64, 1000, 4097};
    const uint32_t ks[] = {1, 2, 3, 8, 32};
    for (size_t si = 0; si < sizeof sizes / sizeof *sizes; ++si) {
        const uint64_t n = sizes[si];
        for (size_t ki = 0; ki < sizeof ks / sizeof *ks; ++ki) {
            const uint32_t k = ks[ki];
            const int wild = (si + ki) % 3 == 0;   /* any bit pattern: NaN, Inf, subnormals */
            uint16_t **parts = (uint16_t **)room(k * sizeof *parts);
            for (uint32_t j = 0; j < k; ++j) {
                parts[j] = (uint16_t *)room(n * 2);
                for (uint64_t i = 0; i < n; ++i) {
                    float f = some_float(wild);
                    uint32_t u;
                    memcpy(&u, &f, 4);
                    parts[j][i] = (uint16_t)(u >> 16);
                }
            }
            float *p = (float *)room(n * 4), *m = (float *)room(n * 4), *v = (float *)room(n * 4);
            for (uint64_t i = 0; i < n; ++i) {
                p[i] = some_float(wild);
                m[i] = some_float(wild) * 1e-3f;
                v[i] = some_float(0);
                v[i] = v[i] < 0 ? -v[i] : v[i];
            }
            double *G = (double *)room(n * 8), *p1 = (double *)room(n * 8), *m1 = (double *)room(n * 8), *v1 = (double *)room(n * 8);
            amsp_oracle_reduce((const uint16_t *const *)parts, k, n, G);
            const double S = amsp_oracle_sqnorm(G, n);
            const double scale = amsp_oracle_clip_scale(S, ki % 2 ? 1.0 : 0.0, 1e-6);
            amsp_oracle_adamw(G, scale, p, m, v, n, 3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, (uint32_t)(1 + si * 7 + ki), p1, m1, v1);
            float *pf = (float *)room(n * 4);
            uint16_t *bf = (uint16_t *)room(n * 2);
            uint8_t *codes = (uint8_t *)room(n);
            amsp_oracle_round_f32(p1, n, pf);
            amsp_oracle_cast(pf, n, bf);
            const float amax = amsp_oracle_absmax(pf, n);
            const float fscale = amsp_oracle_fp8_scale(amax);
            amsp_oracle_cast_fp8(pf, n, fscale, codes);
            uint64_t h = 0xCBF29CE484222325ull;
            h = fnv(G, n * 8, h); h = fnv(&S, 8, h); h = fnv(&scale, 8, h);
            h = fnv(p1, n * 8, h); h = fnv(m1, n * 8, h); h = fnv(v1, n * 8, h);
            h = fnv(pf, n * 4, h); h = fnv(bf, n * 2, h); h = fnv(&amax, 4, h); h = fnv(&fscale, 4, h); h = fnv(codes, n, h);
            printf("n=%llu k=%u wild=%d %016llx\n", (unsigned long long)n, k, wild, (unsigned long long)h);
            for (uint32_t j = 0; j < k; ++j) free(parts[j]);
            free(parts); free(p); free(m); free(v); free(G); free(p1); free(m1); free(v1); free(pf); free(bf); free(codes);
        }
    }
    /* scalar functions over every pattern class */
    uint64_t h = 0xCBF29CE484222325ull;
    for (uint32_t hi = 0; hi < 65536; ++hi) {
        const uint32_t lows[] = {0x0000u, 0x0001u, 0x7FFFu, 0x8000u, 0x8001u, 0xFFFFu};
        for (int l = 0; l < 6; ++l) {
            const uint32_t u = (hi << 16) | lows[l];
            float f;
            memcpy(&f, &u, 4);
            const uint16_t b = amsp_oracle_bf16_rne(f);
            const uint8_t c = amsp_oracle_e4m3_encode(f);
            h = fnv(&b, 2, h); h = fnv(&c, 1, h);
        }
    }
    for (int c = 0; c < 256; ++c) { const float f = amsp_oracle_e4m3_decode((uint8_t)c); h = fnv(&f, 4, h); }
    for (int t = 0; t < 2000; ++t) {
        uint64_t b, e;
        const uint32_t s = 1 + (uint32_t)(rnd() % 100000);
        const uint64_t total = rnd();          /* one draw per statement: the order of evaluation of */
        const unsigned shift = (unsigned)(rnd() % 40);   /* function arguments is unspecified */
        const uint32_t r = (uint32_t)(rnd() % s);
        amsp_oracle_shard_range(total >> shift, s, r, &b, &e);
        h = fnv(&b, 8, h); h = fnv(&e, 8, h);
    }
    printf("scalars %016llx\n", (unsigned long long)h);
    return 0;
}
