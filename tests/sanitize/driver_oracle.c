/* Runs every entry point of the C oracle on small inputs under AddressSanitizer and
 * UndefinedBehaviorSanitizer (the oracle source is compiled into this program with
 * -fsanitize=address,undefined).  Shapes cover empty sequences, one-token sequences, grouped
 * heads, key shards with rows that see nothing, and every element size of the permute.
 * Exit status 0 = every call returned as expected; the sanitizers abort on a finding. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int flexsp_oracle_attn(const void *, const void *, const void *, const void *, int, const int32_t *, int, int, int, int,
                       int, double, double *, double *, double *, double *, double *);
int flexsp_oracle_rows(const void *, const void *, const void *, const void *, int, const int32_t *, int, int, int, int,
                       int, double, const int64_t *, const int32_t *, int, double *, double *, double *);
int flexsp_oracle_dkv_rows(const void *, const void *, const void *, const void *, int, const int32_t *, int, int, int,
                           int, int, double, const int32_t *, const int32_t *, const int32_t *, const int32_t *, int,
                           double *, double *);
int flexsp_oracle_attn_kvshard(const void *, const void *, const void *, int, const int32_t *, const int32_t *,
                               const int32_t *, int, int, int, int, int, double, double *, double *);
int flexsp_oracle_pack(const void *, void *, int64_t, int, int, int, int);
int flexsp_oracle_unpack(const void *, void *, int64_t, int, int, int, int);

static uint16_t *rand_bf16(size_t n, unsigned seed)
{
    uint16_t *p = malloc((n ? n : 1) * sizeof(uint16_t));
    for (size_t i = 0; i < n; i++) {
        seed = seed * 1664525u + 1013904223u;
        float f = ((float)(seed >> 8) / 8388608.0f) - 1.0f;
        uint32_t u;
        __builtin_memcpy(&u, &f, 4);
        p[i] = (uint16_t)(u >> 16);
    }
    return p;
}

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "FAILED: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main(void)
{
    for (int causal = 0; causal < 2; causal++) {
        const int32_t cu[] = {0, 0, 1, 18, 18, 50};
        const int B = 5, T = 50, Hq = 4, Hkv = 2, D = 8;
        uint16_t *q = rand_bf16((size_t)T * Hq * D, 1), *k = rand_bf16((size_t)T * Hkv * D, 2);
        uint16_t *v = rand_bf16((size_t)T * Hkv * D, 3), *g = rand_bf16((size_t)T * Hq * D, 4);
        double *O = malloc(sizeof(double) * T * Hq * D), *L = malloc(sizeof(double) * Hq * T);
        double *dQ = malloc(sizeof(double) * T * Hq * D), *dK = malloc(sizeof(double) * T * Hkv * D);
        double *dV = malloc(sizeof(double) * T * Hkv * D);
        CHECK(flexsp_oracle_attn(q, k, v, g, 1, cu, B, Hq, Hkv, D, causal, 0.35, O, L, dQ, dK, dV) == 0);
        CHECK(flexsp_oracle_attn(q, k, v, NULL, 1, cu, B, Hq, Hkv, D, causal, 0.35, O, L, NULL, NULL, NULL) == 0);
        for (int i = 0; i < T * Hq * D; i++) CHECK(isfinite(O[i]) && isfinite(dQ[i]));
        const int64_t tok[] = {1, 2, 17, 18, 49};
        const int32_t head[] = {0, 3, 1, 2, 3};
        double Or[5 * 8], Lr[5], dQr[5 * 8];
        CHECK(flexsp_oracle_rows(q, k, v, g, 1, cu, B, Hq, Hkv, D, causal, 0.35, tok, head, 5, Or, Lr, dQr) == 0);
        for (int n = 0; n < 5; n++)
            for (int d = 0; d < D; d++) CHECK(fabs(Or[n * D + d] - O[(tok[n] * Hq + head[n]) * D + d]) < 1e-12);
        const int32_t seq[] = {2, 4, 1}, kvh[] = {0, 1, 1}, joff[] = {0, 2, 5, 6}, jl[] = {0, 16, 0, 7, 31, 0};
        double dKr[6 * 8], dVr[6 * 8];
        CHECK(flexsp_oracle_dkv_rows(q, k, v, g, 1, cu, B, Hq, Hkv, D, causal, 0.35, seq, kvh, joff, jl, 3, dKr, dVr) == 0);
        CHECK(fabs(dKr[0] - dK[((cu[2] + 0) * Hkv + 0) * D]) < 1e-12);
        CHECK(fabs(dVr[2 * D + 1] - dV[((cu[4] + 0) * Hkv + 1) * D + 1]) < 1e-12);
        /* key shards: keys of every sequence cut in two, second shard starts at cut[b] */
        const int32_t cu_k[] = {0, 0, 1, 9, 9, 20}, shift[] = {0, 0, 3, 0, -21};
        double *Os = malloc(sizeof(double) * T * Hq * D), *Ls = malloc(sizeof(double) * Hq * T);
        CHECK(flexsp_oracle_attn_kvshard(q, k, v, 1, cu, cu_k, shift, B, Hq, Hkv, D, causal, 0.35, Os, Ls) == 0);
        if (causal) CHECK(isinf(Ls[0 * T + 18]) && Os[(18 * Hq + 0) * D] == 0.0); /* row 0 of the last sequence sees keys <= -21 */
        /* bad arguments are refused, not dereferenced */
        const int32_t bad[] = {0, 5, 3};
        CHECK(flexsp_oracle_attn(q, k, v, g, 1, bad, 2, Hq, Hkv, D, causal, 0.35, O, L, dQ, dK, dV) == -1);
        CHECK(flexsp_oracle_attn(q, k, v, g, 1, cu, B, 3, 2, D, causal, 0.35, O, L, dQ, dK, dV) == -1);
        free(q); free(k); free(v); free(g); free(O); free(L); free(dQ); free(dK); free(dV); free(Os); free(Ls);
    }
    for (int eb = 1; eb <= 16; eb *= 2) {
        const int T = 7, H = 6, D = 5, P = 3;
        unsigned char *x = malloc((size_t)T * H * D * eb), *y = malloc((size_t)T * H * D * eb), *z = malloc((size_t)T * H * D * eb);
        for (int i = 0; i < T * H * D * eb; i++) x[i] = (unsigned char)(i * 37 + eb);
        CHECK(flexsp_oracle_pack(x, y, T, H, D, P, eb) == 0);
        CHECK(flexsp_oracle_unpack(y, z, T, H, D, P, eb) == 0);
        for (int i = 0; i < T * H * D * eb; i++) CHECK(x[i] == z[i]);
        CHECK(flexsp_oracle_pack(x, y, T, H, D, 4, eb) == -1);
        CHECK(flexsp_oracle_pack(x, y, 0, H, D, P, eb) == 0);
        free(x); free(y); free(z);
    }
    puts("oracle under sanitizers: ok");
    return 0;
}
