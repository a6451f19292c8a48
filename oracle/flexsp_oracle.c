/*
 * CPU fp64 oracle for packed (varlen) multi-head attention, forward and backward,
 * and for the sequence-sharded <-> head-sharded layout permute.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is deliberately plain and slow.  It shares no
 * code with the HIP library; only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.
 *
 * What it computes (paper Sec. 2.1.2, Eq. 3: softmax(Q K^T / sqrt(d)) V evaluated
 * on complete sequences for the heads a device holds; Sec. 2.2.2 "Sequence
 * Packing": sequences concatenated into one stream must not see each other):
 *
 *   for every sequence b (tokens cu[b] .. cu[b+1]-1), query head h, kv head g = h / G,
 *   row i of the sequence, with J(i) = {0..i} (causal) or {0..s-1}:
 *     S_ij  = scale * sum_d q[i,h,d] k[j,g,d]
 *     m_i   = max_j S_ij ;  Z_i = sum_j exp(S_ij - m_i)
 *     P_ij  = exp(S_ij - m_i) / Z_i ;  LSE_i = m_i + ln Z_i
 *     O_i   = sum_j P_ij v[j,g,:]
 *   and, for an upstream gradient dO (gradient of L = sum O .* dO):
 *     dP_ij = sum_d dO[i,h,d] v[j,g,d]
 *     delta_i = sum_j P_ij dP_ij
 *     dS_ij = P_ij (dP_ij - delta_i)
 *     dQ[i,h,:] = scale * sum_j dS_ij k[j,g,:]
 *     dK[j,g,:] = scale * sum_{h in group(g)} sum_i dS_ij q[i,h,:]
 *     dV[j,g,:] =         sum_{h in group(g)} sum_i P_ij  dO[i,h,:]
 *
 * Every sum is a sequential fp64 sum in index order.  One row of S is materialised
 * at a time.  No tiling, no online softmax.  The only layout liberty: K and V of
 * the (sequence, kv-head) at hand are also copied transposed so that the inner loop
 * of the dot products runs over j (each S_ij is still summed over d in order).
 *
 * Inputs are either fp64 arrays (dtype 0) or bf16 bit patterns (dtype 1, uint16),
 * the latter widened exactly to fp64.  Layouts: q, dO, O, dQ [T, Hq, D];
 * k, v, dK, dV [T, Hkv, D]; LSE [Hq, T]; all row-major, last dim contiguous.
 *
 * The layout permute (the local half of the exchanges in Eq. 2 and Eq. 4):
 *   pack:   dst[r, t, h, :] = src[t, r*(H/P) + h, :]
 *   unpack: dst[t, r*(H/P) + h, :] = src[r, t, h, :]
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == 0)
        return ((const double *)base)[idx];
    uint32_t u = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* copy rows [t0, t0+s) of head h of x[T,H,D] into dst[s,D] (fp64) */
static void gather(const void *x, int dtype, int64_t t0, int s, int H, int h, int D, double *dst)
{
    for (int i = 0; i < s; i++)
        for (int d = 0; d < D; d++)
            dst[(int64_t)i * D + d] = widen(x, dtype, ((t0 + i) * H + h) * D + d);
}

static void transpose(const double *x, int s, int D, double *xt)
{
    for (int i = 0; i < s; i++)
        for (int d = 0; d < D; d++)
            xt[(int64_t)d * s + i] = x[(int64_t)i * D + d];
}

/* One row: scores, softmax, output.  kt = K transposed [D,s].  Returns n = |J(i)|.
 * p (length >= n) receives the probabilities. */
static int row_forward(const double *qi, const double *kt, const double *v, int s, int D, int i,
                       int causal, double scale, double *p, double *o, double *lse)
{
    int n = causal ? i + 1 : s;
    for (int j = 0; j < n; j++) p[j] = 0.0;
    for (int d = 0; d < D; d++) {
        double qd = qi[d];
        const double *kr = kt + (int64_t)d * s;
        for (int j = 0; j < n; j++) p[j] += qd * kr[j];
    }
    double m = -INFINITY;
    for (int j = 0; j < n; j++) {
        p[j] *= scale;
        if (p[j] > m) m = p[j];
    }
    double z = 0.0;
    for (int j = 0; j < n; j++) {
        p[j] = exp(p[j] - m);
        z += p[j];
    }
    for (int j = 0; j < n; j++) p[j] /= z;
    if (lse) *lse = m + log(z);
    if (o) {
        for (int d = 0; d < D; d++) o[d] = 0.0;
        for (int j = 0; j < n; j++) {
            const double *vj = v + (int64_t)j * D;
            double pj = p[j];
            for (int d = 0; d < D; d++) o[d] += pj * vj[d];
        }
    }
    return n;
}

/* dP row, delta, dS row (written over dp).  vt = V transposed [D,s]. */
static double row_backward(const double *doi, const double *vt, int s, int D, int n,
                           const double *p, double *ds)
{
    for (int j = 0; j < n; j++) ds[j] = 0.0;
    for (int d = 0; d < D; d++) {
        double g = doi[d];
        const double *vr = vt + (int64_t)d * s;
        for (int j = 0; j < n; j++) ds[j] += g * vr[j];
    }
    double delta = 0.0;
    for (int j = 0; j < n; j++) delta += p[j] * ds[j];
    for (int j = 0; j < n; j++) ds[j] = p[j] * (ds[j] - delta);
    return delta;
}

typedef struct {
    double *q, *k, *v, *g, *kt, *vt, *p, *ds;
} scratch_t;

static int scratch_alloc(scratch_t *w, int s, int D)
{
    size_t n = (size_t)s * D;
    if (n == 0) n = 1;
    w->q = malloc(n * 8); w->k = malloc(n * 8); w->v = malloc(n * 8); w->g = malloc(n * 8);
    w->kt = malloc(n * 8); w->vt = malloc(n * 8);
    w->p = malloc((size_t)(s + 1) * 8); w->ds = malloc((size_t)(s + 1) * 8);
    return (w->q && w->k && w->v && w->g && w->kt && w->vt && w->p && w->ds) ? 0 : -1;
}

static void scratch_free(scratch_t *w)
{
    free(w->q); free(w->k); free(w->v); free(w->g); free(w->kt); free(w->vt); free(w->p); free(w->ds);
}

static int check_dims(int B, int Hq, int Hkv, int D, const int32_t *cu)
{
    if (B < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv) return -1;
    if (cu[0] != 0) return -1;
    for (int b = 0; b < B; b++)
        if (cu[b + 1] < cu[b]) return -1;
    return 0;
}

/*
 * Full forward (+ optional backward when dO != NULL) over the packed batch.
 * Outputs are fp64: O [T,Hq,D], LSE [Hq,T]; dQ [T,Hq,D], dK, dV [T,Hkv,D] (may be
 * NULL together with dO).  Parallel over (sequence, kv head) only; inside one such
 * pair everything is sequential, so thread count never changes a value.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int flexsp_oracle_attn(const void *q, const void *k, const void *v, const void *dO, int dtype,
                       const int32_t *cu, int B, int Hq, int Hkv, int D, int causal, double scale,
                       double *O, double *LSE, double *dQ, double *dK, double *dV)
{
    if (check_dims(B, Hq, Hkv, D, cu)) return -1;
    int G = Hq / Hkv;
    int64_t T = cu[B];
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; b++) {
        for (int g = 0; g < Hkv; g++) {
            int64_t t0 = cu[b];
            int s = cu[b + 1] - cu[b];
            if (s == 0) continue;
            scratch_t w;
            if (scratch_alloc(&w, s, D)) { failed = 1; scratch_free(&w); continue; }
            gather(k, dtype, t0, s, Hkv, g, D, w.k);
            gather(v, dtype, t0, s, Hkv, g, D, w.v);
            transpose(w.k, s, D, w.kt);
            transpose(w.v, s, D, w.vt);
            if (dO) {
                for (int i = 0; i < s; i++)
                    for (int d = 0; d < D; d++) {
                        dK[((t0 + i) * Hkv + g) * D + d] = 0.0;
                        dV[((t0 + i) * Hkv + g) * D + d] = 0.0;
                    }
            }
            for (int hh = 0; hh < G; hh++) {
                int h = g * G + hh;
                gather(q, dtype, t0, s, Hq, h, D, w.q);
                if (dO) gather(dO, dtype, t0, s, Hq, h, D, w.g);
                for (int i = 0; i < s; i++) {
                    const double *qi = w.q + (int64_t)i * D;
                    double *oi = O + ((t0 + i) * Hq + h) * D;
                    int n = row_forward(qi, w.kt, w.v, s, D, i, causal, scale, w.p, oi,
                                        &LSE[(int64_t)h * T + t0 + i]);
                    if (!dO) continue;
                    const double *gi = w.g + (int64_t)i * D;
                    row_backward(gi, w.vt, s, D, n, w.p, w.ds);
                    double *dqi = dQ + ((t0 + i) * Hq + h) * D;
                    for (int d = 0; d < D; d++) dqi[d] = 0.0;
                    for (int j = 0; j < n; j++) {
                        const double *kj = w.k + (int64_t)j * D;
                        double *dkj = dK + ((t0 + j) * Hkv + g) * D;
                        double *dvj = dV + ((t0 + j) * Hkv + g) * D;
                        double dsj = w.ds[j], pj = w.p[j];
                        for (int d = 0; d < D; d++) {
                            dqi[d] += dsj * kj[d];
                            dkj[d] += dsj * qi[d];
                            dvj[d] += pj * gi[d];
                        }
                    }
                    for (int d = 0; d < D; d++) dqi[d] *= scale;
                }
            }
            if (dO) {
                for (int i = 0; i < s; i++)
                    for (int d = 0; d < D; d++) dK[((t0 + i) * Hkv + g) * D + d] *= scale;
            }
            scratch_free(&w);
        }
    }
    return failed ? -1 : 0;
}

static int find_seq(const int32_t *cu, int B, int64_t t)
{
    for (int b = 0; b < B; b++)
        if (t >= cu[b] && t < cu[b + 1]) return b;
    return -1;
}

/*
 * Sampled rows of O / LSE / dQ: for sample n the pair (tok[n], head[n]) names a token of
 * the packed stream and a query head.  O_rows, dQ_rows [N,D]; LSE_rows [N].  dO, dQ_rows
 * may be NULL together.  Cost per sample is O(i D) for a row i of its sequence.
 */
int flexsp_oracle_rows(const void *q, const void *k, const void *v, const void *dO, int dtype,
                       const int32_t *cu, int B, int Hq, int Hkv, int D, int causal, double scale,
                       const int64_t *tok, const int32_t *head, int N,
                       double *O_rows, double *LSE_rows, double *dQ_rows)
{
    if (check_dims(B, Hq, Hkv, D, cu)) return -1;
    int G = Hq / Hkv;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < N; n++) {
        int b = find_seq(cu, B, tok[n]);
        int h = head[n];
        if (b < 0 || h < 0 || h >= Hq) { failed = 1; continue; }
        int g = h / G;
        int64_t t0 = cu[b];
        int s = cu[b + 1] - cu[b];
        int i = (int)(tok[n] - t0);
        int m = causal ? i + 1 : s; /* only keys 0..m-1 matter */
        scratch_t w;
        if (scratch_alloc(&w, m, D)) { failed = 1; scratch_free(&w); continue; }
        gather(k, dtype, t0, m, Hkv, g, D, w.k);
        gather(v, dtype, t0, m, Hkv, g, D, w.v);
        transpose(w.k, m, D, w.kt);
        transpose(w.v, m, D, w.vt);
        gather(q, dtype, t0 + i, 1, Hq, h, D, w.q);
        /* with causal masking row i of the length-m prefix is row i of the sequence */
        int cnt = row_forward(w.q, w.kt, w.v, m, D, causal ? i : 0, causal, scale, w.p,
                              O_rows + (int64_t)n * D, &LSE_rows[n]);
        if (dO && dQ_rows) {
            gather(dO, dtype, t0 + i, 1, Hq, h, D, w.g);
            row_backward(w.g, w.vt, m, D, cnt, w.p, w.ds);
            double *dqi = dQ_rows + (int64_t)n * D;
            for (int d = 0; d < D; d++) dqi[d] = 0.0;
            for (int j = 0; j < cnt; j++)
                for (int d = 0; d < D; d++) dqi[d] += w.ds[j] * w.k[(int64_t)j * D + d];
            for (int d = 0; d < D; d++) dqi[d] *= scale;
        }
        scratch_free(&w);
    }
    return failed ? -1 : 0;
}

/*
 * Sampled rows of dK / dV.  Task n names a sequence seq[n], a kv head kvh[n] and a list of
 * key positions inside that sequence, jlist[joff[n] .. joff[n+1]) (ascending).  Rows
 * i >= min(j) of every query head of the group are evaluated once each and accumulated
 * into every listed j <= i (all j when not causal: then every row is evaluated).
 * dK_rows, dV_rows [joff[N], D].
 */
int flexsp_oracle_dkv_rows(const void *q, const void *k, const void *v, const void *dO, int dtype,
                           const int32_t *cu, int B, int Hq, int Hkv, int D, int causal,
                           double scale, const int32_t *seq, const int32_t *kvh,
                           const int32_t *joff, const int32_t *jlist, int N,
                           double *dK_rows, double *dV_rows)
{
    if (check_dims(B, Hq, Hkv, D, cu)) return -1;
    int G = Hq / Hkv;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < N; n++) {
        int b = seq[n], g = kvh[n];
        int nj = joff[n + 1] - joff[n];
        if (b < 0 || b >= B || g < 0 || g >= Hkv || nj <= 0) { failed = 1; continue; }
        const int32_t *js = jlist + joff[n];
        int64_t t0 = cu[b];
        int s = cu[b + 1] - cu[b];
        int jmin = js[0];
        for (int a = 0; a < nj; a++) {
            if (js[a] < 0 || js[a] >= s) failed = 1;
            if (js[a] < jmin) jmin = js[a];
        }
        if (failed) continue;
        scratch_t w;
        if (scratch_alloc(&w, s, D)) { failed = 1; scratch_free(&w); continue; }
        gather(k, dtype, t0, s, Hkv, g, D, w.k);
        gather(v, dtype, t0, s, Hkv, g, D, w.v);
        transpose(w.k, s, D, w.kt);
        transpose(w.v, s, D, w.vt);
        double *dk = dK_rows + (int64_t)joff[n] * D;
        double *dv = dV_rows + (int64_t)joff[n] * D;
        for (int64_t e = 0; e < (int64_t)nj * D; e++) dk[e] = dv[e] = 0.0;
        int ifirst = causal ? jmin : 0;
        for (int hh = 0; hh < G; hh++) {
            int h = g * G + hh;
            for (int i = ifirst; i < s; i++) {
                gather(q, dtype, t0 + i, 1, Hq, h, D, w.q);
                gather(dO, dtype, t0 + i, 1, Hq, h, D, w.g);
                int cnt = row_forward(w.q, w.kt, w.v, s, D, i, causal, scale, w.p, NULL, NULL);
                row_backward(w.g, w.vt, s, D, cnt, w.p, w.ds);
                for (int a = 0; a < nj; a++) {
                    int j = js[a];
                    if (j >= cnt) continue;
                    for (int d = 0; d < D; d++) {
                        dk[(int64_t)a * D + d] += w.ds[j] * w.q[d];
                        dv[(int64_t)a * D + d] += w.p[j] * w.g[d];
                    }
                }
            }
        }
        for (int64_t e = 0; e < (int64_t)nj * D; e++) dk[e] *= scale;
        scratch_free(&w);
    }
    return failed ? -1 : 0;
}

/*
 * Attention of each sequence's queries against ONE SHARD of its keys, the unit of work of context
 * parallelism (paper Sec. 2.1.3, paragraph "Context Parallelism": queries, keys and values are split along
 * the sequence, key/value chunks travel round a ring, and attention is computed chunk by chunk;
 * the appendix on integrating context parallelism).  Sequence b has queries at rows
 * cu_q[b] .. cu_q[b+1]-1 of q and shard keys at rows cu_k[b] .. cu_k[b+1]-1 of k and v.  With
 * causal masking, shard key j is visible to query i iff j <= i + shift[b], where shift[b] =
 * (position of the first query in its sequence) - (position of the shard's first key); without,
 * every shard key is visible.  Per row: softmax over the visible shard keys only,
 *   O_i = sum_j P_ij v_j,  LSE_i = log sum_j exp(S_ij);   no visible key: O_i = 0, LSE_i = -inf.
 * The visible keys of a row are always a prefix 0 .. n-1 of the shard, so a row is evaluated by
 * row_forward as the last row of a causal problem over that prefix: no new arithmetic.
 * O [Tq, Hq, D], LSE [Hq, Tq], fp64.
 */
int flexsp_oracle_attn_kvshard(const void *q, const void *k, const void *v, int dtype, const int32_t *cu_q,
                               const int32_t *cu_k, const int32_t *shift, int B, int Hq, int Hkv, int D,
                               int causal, double scale, double *O, double *LSE)
{
    if (check_dims(B, Hq, Hkv, D, cu_q) || check_dims(B, Hq, Hkv, D, cu_k)) return -1;
    int G = Hq / Hkv;
    int64_t Tq = cu_q[B];
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; b++) {
        for (int g = 0; g < Hkv; g++) {
            int64_t tq0 = cu_q[b], tk0 = cu_k[b];
            int sq = cu_q[b + 1] - cu_q[b], sk = cu_k[b + 1] - cu_k[b];
            if (sq == 0) continue;
            scratch_t w;
            int m = sk > sq ? sk : sq;
            if (scratch_alloc(&w, m, D)) { failed = 1; scratch_free(&w); continue; }
            gather(k, dtype, tk0, sk, Hkv, g, D, w.k);
            gather(v, dtype, tk0, sk, Hkv, g, D, w.v);
            transpose(w.k, sk, D, w.kt);
            for (int hh = 0; hh < G; hh++) {
                int h = g * G + hh;
                gather(q, dtype, tq0, sq, Hq, h, D, w.q);
                for (int i = 0; i < sq; i++) {
                    int64_t n = causal ? (int64_t)i + shift[b] + 1 : sk; /* visible keys: 0 .. n-1 */
                    if (n > sk) n = sk;
                    double *oi = O + ((tq0 + i) * Hq + h) * D;
                    double *li = &LSE[(int64_t)h * Tq + tq0 + i];
                    if (n <= 0) {
                        for (int d = 0; d < D; d++) oi[d] = 0.0;
                        *li = -INFINITY;
                        continue;
                    }
                    row_forward(w.q + (int64_t)i * D, w.kt, w.v, sk, D, (int)n - 1, 1, scale, w.p, oi, li);
                }
            }
            scratch_free(&w);
        }
    }
    return failed ? -1 : 0;
}

/* Layout permute on raw elements of `eb` bytes each.  Requires H % P == 0. */
int flexsp_oracle_pack(const void *src, void *dst, int64_t T, int H, int D, int P, int eb)
{
    if (T < 0 || H <= 0 || D <= 0 || P <= 0 || eb <= 0 || H % P) return -1;
    int Hp = H / P;
    const char *s = src;
    char *o = dst;
    for (int r = 0; r < P; r++)
        for (int64_t t = 0; t < T; t++)
            for (int h = 0; h < Hp; h++)
                for (int d = 0; d < D; d++)
                    memcpy(o + ((((int64_t)r * T + t) * Hp + h) * D + d) * eb,
                           s + ((t * H + (int64_t)r * Hp + h) * D + d) * eb, eb);
    return 0;
}

int flexsp_oracle_unpack(const void *src, void *dst, int64_t T, int H, int D, int P, int eb)
{
    if (T < 0 || H <= 0 || D <= 0 || P <= 0 || eb <= 0 || H % P) return -1;
    int Hp = H / P;
    const char *s = src;
    char *o = dst;
    for (int64_t t = 0; t < T; t++)
        for (int hh = 0; hh < H; hh++) {
            int r = hh / Hp, h = hh % Hp;
            for (int d = 0; d < D; d++)
                memcpy(o + ((t * H + hh) * D + d) * eb,
                       s + ((((int64_t)r * T + t) * Hp + h) * D + d) * eb, eb);
        }
    return 0;
}
