/*
 * CTkvr CPU oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * A plain, slow implementation of the centroid-then-token KV retrieval of the
 * CTkvr paper, written from the paper's Algorithm 1 (index construction at
 * prefill, lines 1-4) and Algorithm 2 (retrieval at decoding, lines 1-9), one
 * step per loop, in the paper's order and notation.  It is used only by the
 * tests, by the smoke check and by the benchmark's reported CPU baseline; the
 * GPU library never links or calls it and shares no code with it.
 *
 * Layout follows the paper's problem statement: per sequence, keys and values
 * K, V in [g][s][d], queries in [h][d], query centroids Q^(c) in [h][C][d],
 * the inverted file qcIVF in [g][C][rho] (int32 key ids).  Query heads
 * h_i = i*h/g .. (i+1)*h/g - 1 share KV head i (footnote on grouped-query
 * attention in Section 3.1.1).
 *
 * Precision.  Every quantity that DECIDES AN INTEGER (which centroids are
 * probed, which keys enter a list, which keys survive the rerank) is computed
 * in one fixed fp32 arithmetic, written out below, so that an independent GPU
 * implementation can reach the same integers bit for bit:
 *   - dot product over d = 128: 16 partial sums, partial l = sequential fmaf
 *     over elements 8l..8l+7 starting from 0, then a balanced pairwise tree
 *     (l, l+1), (l, l+2), (l, l+4), (l, l+8);
 *   - 1/norm = 1.0f / sqrtf(dot(x, x))  (IEEE sqrt and divide; 0 if dot = 0);
 *   - the softmax of Algorithm 1 line 2 and Algorithm 2 line 5 is ranked in
 *     the log domain: log softmax_i = (z_i - m) - log(sum_j exp(z_j - m)); the
 *     sum is accumulated in 2^-40 fixed point (integer adds, hence the same
 *     value in any order), exp and log are the short series below.
 *     Ranking by log-softmax equals ranking by softmax (log is increasing).
 * The attention output (Algorithm 2 line 9) decides no integer and is
 * computed in fp64 from the inputs.
 *
 * Ties: lowest id wins (centroid id in the probe selection, key id in the
 * list and rerank selections).  Sets are stored in ascending id order.
 *
 * Pins: tests/test_oracle_*.py check this file against brute-force dense
 * attention, brute-force fp64 definitions on small inputs, closed forms the
 * paper prints, and library exp/log/sort -- none of them calls back into it.
 * The k-means centroid mode at the end of the file has pins of its own
 * (tests/test_oracle_kmeans.py, listed in its header).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define D 128            /* head dimension the path is specified for */
#define FIX_SHIFT 40     /* fixed-point position of the softmax denominator */

/* ------------------------------------------------------------------------- */
/* fixed fp32 arithmetic                                                      */
/* ------------------------------------------------------------------------- */
float ctkvr_oracle_dot128(const float *a, const float *b)
{
    float p[16];
    for (int l = 0; l < 16; ++l) {
        float acc = 0.0f;
        for (int e = 0; e < 8; ++e)
            acc = fmaf(a[8 * l + e], b[8 * l + e], acc);
        p[l] = acc;
    }
    for (int m = 1; m < 16; m *= 2)
        for (int l = 0; l < 16; l += 2 * m)
            p[l] = p[l] + p[l + m];
    return p[0];
}

float ctkvr_oracle_inv_norm(const float *x)
{
    float n2 = ctkvr_oracle_dot128(x, x);
    if (!(n2 > 0.0f))
        return 0.0f;
    return 1.0f / sqrtf(n2);
}

/* exp(x) for x <= 0, fp32, fmaf only.  x = n ln2 + r, |r| <= ln2/2, degree-7
 * Taylor polynomial of exp(r) (remainder < 6e-9 relative), scaled by 2^n.
 * Below -30 the value is < 2^-43 and contributes nothing at 2^-40 resolution:
 * defined as 0. */
float ctkvr_oracle_exp(float x)
{
    if (!(x >= -30.0f))
        return 0.0f;
    const float MAGIC = 12582912.0f;                 /* 1.5 * 2^23: round to nearest integer */
    float t = fmaf(x, 1.44269504088896341f, MAGIC);
    float n = t - MAGIC;
    float r = fmaf(n, -0.693145751953125f, x);       /* ln2 high part (exact product with |n| < 2^8) */
    r = fmaf(n, -1.42860682030941723e-6f, r);        /* ln2 low part */
    float p = 1.0f / 5040.0f;
    p = fmaf(p, r, 1.0f / 720.0f);
    p = fmaf(p, r, 1.0f / 120.0f);
    p = fmaf(p, r, 1.0f / 24.0f);
    p = fmaf(p, r, 1.0f / 6.0f);
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    union { uint32_t u; float f; } two_n;
    two_n.u = (uint32_t)((int32_t)n + 127) << 23;
    return p * two_n.f;
}

/* floor(e * 2^40) for 0 <= e < 2 as an integer (the product is exact in fp64) */
static uint64_t to_fixed(float e)
{
    return (uint64_t)((double)e * 1099511627776.0);
}

/* log(S * 2^-40) for an integer S >= 1, fp64: S = 2^k f with f in
 * [sqrt(1/2), sqrt(2)); log f = 2 atanh(u), u = (f-1)/(f+1), odd series to
 * u^23 (|u| < 0.1716, truncation < 1e-18). */
double ctkvr_oracle_log_fixed(uint64_t S)
{
    if (S == 0)
        return -INFINITY;
    int k = 63;
    while (!((S >> k) & 1))
        --k;
    /* top 53 bits, truncated (exact unless S >= 2^53) */
    uint64_t mant = (k > 52) ? (S >> (k - 52)) : (S << (52 - k));
    double f = (double)mant * 0x1p-52;              /* in [1, 2) */
    if (f > 1.4142135623730951) {
        f = f * 0.5;
        k += 1;
    }
    double u = (f - 1.0) / (f + 1.0);
    double u2 = u * u;
    double p = 1.0 / 23.0;
    for (int q = 21; q >= 1; q -= 2)
        p = fma(p, u2, 1.0 / (double)q);
    return fma((double)(k - FIX_SHIFT), 0.6931471805599453, 2.0 * u * p);
}

/* ------------------------------------------------------------------------- */
/* selection helpers: top-n by (score descending, id ascending)               */
/* ------------------------------------------------------------------------- */
typedef struct { float score; int32_t id; } scored;

static int cmp_scored(const void *pa, const void *pb)
{
    const scored *a = (const scored *)pa, *b = (const scored *)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

static int cmp_i32(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/* ids of the n best of (score[i], id[i]), written in ascending id order */
static void top_n_ids(const float *score, const int32_t *id, int count, int n, int32_t *out)
{
    scored *w = (scored *)malloc(sizeof(scored) * (size_t)(count > 0 ? count : 1));
    for (int i = 0; i < count; ++i) {
        w[i].score = score[i];
        w[i].id = id ? id[i] : i;
    }
    qsort(w, (size_t)count, sizeof(scored), cmp_scored);
    if (n > count) n = count;
    for (int i = 0; i < n; ++i)
        out[i] = w[i].id;
    qsort(out, (size_t)n, sizeof(int32_t), cmp_i32);
    free(w);
}

/* ------------------------------------------------------------------------- */
/* max_kv-group(Softmax(Q . K^set)) in the log domain                         */
/*   Algorithm 1 lines 2-3 (set = all s keys, Q = a centroid)                 */
/*   Algorithm 2 line 5    (set = recalled keys, Q = the decode query)        */
/* q: G query vectors of one KV group, Kg: [s][D] keys of that KV head.       */
/* key_out[i] = max_h log softmax_h(i) over the L ids in set[].               */
/* ------------------------------------------------------------------------- */
static void group_log_softmax_max(const float *q, int G, const float *Kg, const int32_t *set, int L,
                                  float scale, float *key_out, float *z_out /* [G][L] or NULL */)
{
    if (L <= 0)
        return;
    float *z = (float *)malloc(sizeof(float) * (size_t)L);
    for (int i = 0; i < L; ++i)
        key_out[i] = -INFINITY;
    for (int hh = 0; hh < G; ++hh) {
        float m = -INFINITY;
        for (int i = 0; i < L; ++i) {
            int32_t t = set ? set[i] : i;
            z[i] = ctkvr_oracle_dot128(q + (size_t)hh * D, Kg + (size_t)t * D) * scale;
            if (z[i] > m) m = z[i];
        }
        uint64_t S = 0;
        for (int i = 0; i < L; ++i)
            S += to_fixed(ctkvr_oracle_exp(z[i] - m));
        float ls = (float)ctkvr_oracle_log_fixed(S);
        for (int i = 0; i < L; ++i) {
            float lp = (z[i] - m) - ls;
            if (lp > key_out[i]) key_out[i] = lp;
        }
        if (z_out)
            memcpy(z_out + (size_t)hh * L, z, sizeof(float) * (size_t)L);
    }
    free(z);
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1, lines 2-4: inverted lists                                     */
/* K [g][s][D]; Qc [h][C][D] (line 1: the centroids, already sliced by the    */
/* caller); pairs = n_pairs x (kv head, centroid) to build, or NULL for all   */
/* g*C in order; lists_out [n_pairs][rho] ascending key ids.                  */
/* n_init, n_local (lines 5-6): the first n_init and the last n_local keys    */
/* stay resident with the attention and are left out of the lists; the scores */
/* (line 2) are still a softmax over all s keys.                              */
/* ------------------------------------------------------------------------- */
void ctkvr_oracle_build_lists(const float *K, const float *Qc, int h, int g, int s, int C, int rho, float scale,
                              const int32_t *pairs, int n_pairs, int n_init, int n_local, int32_t *lists_out,
                              float *keys_out /* [n_pairs][s] or NULL */)
{
    int G = h / g;
    if (!pairs) n_pairs = g * C;
#pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < n_pairs; ++p) {
        int kv = pairs ? pairs[2 * p] : p / C;
        int j = pairs ? pairs[2 * p + 1] : p % C;
        float *q = (float *)malloc(sizeof(float) * (size_t)G * D);
        float *key = (float *)malloc(sizeof(float) * (size_t)s);
        for (int hh = 0; hh < G; ++hh)
            memcpy(q + (size_t)hh * D, Qc + ((size_t)(kv * G + hh) * C + j) * D, sizeof(float) * D);
        /* lines 2-3: A_kv[kv, j, :] */
        group_log_softmax_max(q, G, K + (size_t)kv * s * D, NULL, s, scale, key, NULL);
        /* line 4: top-rho, among the keys that leave the resident window */
        int32_t *lst = lists_out + (size_t)p * rho;
        top_n_ids(key + n_init, NULL, s - n_init - n_local, rho, lst);
        for (int r = 0; r < rho; ++r)
            lst[r] += n_init;
        if (keys_out)
            memcpy(keys_out + (size_t)p * s, key, sizeof(float) * (size_t)s);
        free(q);
        free(key);
    }
}

/* inverse norms of n vectors of length D */
void ctkvr_oracle_inv_norms(const float *X, int n, float *out)
{
    for (int i = 0; i < n; ++i)
        out[i] = ctkvr_oracle_inv_norm(X + (size_t)i * D);
}

/* ------------------------------------------------------------------------- */
/* Algorithm 2, lines 1-3: Q2Q^(c) recall -- which centroids are probed       */
/* q [h][D]; Qc [h][C][D]; cos_kv_out [g][C]; probe_out [g][n_probe] asc.     */
/* ------------------------------------------------------------------------- */
void ctkvr_oracle_recall(const float *q, const float *Qc, int h, int g, int C, int n_probe,
                         float *cos_kv_out, int32_t *probe_out)
{
    int G = h / g;
    for (int kv = 0; kv < g; ++kv) {
        float *cosv = cos_kv_out + (size_t)kv * C;
        for (int j = 0; j < C; ++j)
            cosv[j] = -INFINITY;
        for (int hh = 0; hh < G; ++hh) {
            int head = kv * G + hh;
            float inq = ctkvr_oracle_inv_norm(q + (size_t)head * D);
            for (int j = 0; j < C; ++j) {
                const float *c = Qc + ((size_t)head * C + j) * D;
                float cs = (ctkvr_oracle_dot128(q + (size_t)head * D, c) * ctkvr_oracle_inv_norm(c)) * inq;   /* line 1 */
                if (cs > cosv[j]) cosv[j] = cs;                                                             /* line 2 */
            }
        }
        top_n_ids(cosv, NULL, C, n_probe, probe_out + (size_t)kv * n_probe);                                /* line 3 */
    }
}

/* ------------------------------------------------------------------------- */
/* Algorithm 2, lines 4-9 for one sequence, given the probed centroids.       */
/* lists [g][C][rho]: only the probed rows are read.                          */
/* cand_out [g][Lmax], Lmax = min(s, n_probe*rho); ncand_out [g];             */
/* rkey_out [g][Lmax] rerank keys (max over group of log-softmax), optional;  */
/* sel_out [g][top_k] ascending, padded with -1; out [h][D] fp64; lse [h].    */
/* ------------------------------------------------------------------------- */
void ctkvr_oracle_rerank_attend(const float *q, const float *K, const float *V, const int32_t *lists,
                                const int32_t *probe, int h, int g, int s, int C, int rho, int n_probe, int top_k,
                                float scale, int32_t *cand_out, int32_t *ncand_out, float *rkey_out,
                                int32_t *sel_out, double *out, double *lse_out)
{
    int G = h / g;
    long Lmax = (long)n_probe * rho;
    if (Lmax > s) Lmax = s;
#pragma omp parallel for schedule(dynamic, 1)
    for (int kv = 0; kv < g; ++kv) {
        const float *Kg = K + (size_t)kv * s * D;
        const float *Vg = V + (size_t)kv * s * D;
        /* line 4: DedupIdx -- sorted unique union of the probed lists */
        unsigned char *seen = (unsigned char *)calloc((size_t)s, 1);
        for (int p = 0; p < n_probe; ++p) {
            const int32_t *lst = lists + ((size_t)kv * C + probe[(size_t)kv * n_probe + p]) * rho;
            for (int r = 0; r < rho; ++r)
                seen[lst[r]] = 1;
        }
        int32_t *cand = cand_out + (size_t)kv * Lmax;
        int L = 0;
        for (int t = 0; t < s; ++t)
            if (seen[t]) cand[L++] = t;
        free(seen);
        ncand_out[kv] = L;
        /* line 5: max over the group of the softmax over the recalled keys */
        float *key = (float *)malloc(sizeof(float) * (size_t)(L > 0 ? L : 1));
        group_log_softmax_max(q + (size_t)kv * G * D, G, Kg, cand, L, scale, key, NULL);
        if (rkey_out)
            memcpy(rkey_out + (size_t)kv * Lmax, key, sizeof(float) * (size_t)L);
        /* line 6: top-rho' */
        int32_t *sel = sel_out + (size_t)kv * top_k;
        int nsel = top_k < L ? top_k : L;
        top_n_ids(key, cand, L, top_k, sel);
        for (int i = nsel; i < top_k; ++i)
            sel[i] = -1;
        free(key);
        /* lines 7-9: gather K^sparse, V^sparse and attend, fp64 */
        double *zz = (double *)malloc(sizeof(double) * (size_t)(nsel > 0 ? nsel : 1));
        for (int hh = 0; hh < G; ++hh) {
            int head = kv * G + hh;
            const float *qh = q + (size_t)head * D;
            double m = -INFINITY;
            for (int i = 0; i < nsel; ++i) {
                const float *kt = Kg + (size_t)sel[i] * D;
                double acc = 0.0;
                for (int e = 0; e < D; ++e)
                    acc += (double)qh[e] * (double)kt[e];
                zz[i] = acc * (double)scale;
                if (zz[i] > m) m = zz[i];
            }
            double den = 0.0;
            for (int i = 0; i < nsel; ++i)
                den += exp(zz[i] - m);
            double *o = out + (size_t)head * D;
            for (int e = 0; e < D; ++e)
                o[e] = 0.0;
            for (int i = 0; i < nsel; ++i) {
                double w = exp(zz[i] - m) / den;
                const float *vt = Vg + (size_t)sel[i] * D;
                for (int e = 0; e < D; ++e)
                    o[e] += w * (double)vt[e];
            }
            if (lse_out)
                lse_out[head] = nsel > 0 ? m + log(den) : -INFINITY;
        }
        free(zz);
    }
}

int ctkvr_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void ctkvr_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ========================================================================= */
/* k-means centroid mode (replaces Algorithm 1 line 1 only; not in the paper: */
/* the benchmark's index-build configuration asks for Lloyd iterations over   */
/* the post-RoPE prompt queries).  Reading, per sequence and KV head:          */
/*   - a point is one prompt position: the concatenation of the G query-head  */
/*     vectors of the group at that position (G*128 numbers);                  */
/*   - squared-Euclidean Lloyd: assign every point to its nearest centre      */
/*     (ties to the lowest centre id), replace every non-empty centre by the  */
/*     mean of its points; an empty centre keeps its place;                    */
/*   - sums are taken in 2^-20 fixed point (llrint(v * 2^20), exact for bf16   */
/*     values of magnitude >= 2^-13), so they do not depend on the order;      */
/*     mean = (double)sum * 2^-20 / count, rounded to fp32 and then, for bf16  */
/*     data, to bf16 (nearest even): the next assignment reads bf16 centres.   */
/* Distances here are fp64.  (A kernel that scores in fp32 on the matrix cores  */
/* may assign a point differently when two centres tie within its rounding;    */
/* the GPU tests therefore compare one iteration at a time from equal centres, */
/* with such near-ties listed, and check the argmin property of the result.)   */
/* Pins (tests/test_oracle_kmeans.py): one centre = the mean; as many centres  */
/* as distinct points = zero inertia; inertia never increases; scipy's         */
/* kmeans2 step from the same start; lattice points: exact means and their     */
/* bf16 rounding; duplicated centres: every point of the tie goes to the       */
/* lowest id; a centre without members keeps its position; explicit start      */
/* centres = the positions they were read from.                                 */
/* ========================================================================= */
static float round_bf16(float x)
{
    union { float f; uint32_t u; } v;
    v.f = x;
    uint32_t lsb = (v.u >> 16) & 1u;
    v.u += 0x7fffu + lsb;
    v.u &= 0xffff0000u;
    return v.f;
}

/* X [n][dim] points, cent [C][dim] centres (in/out), assign_out [n], inertia_out [iters+1]:
 * inertia_out[i] = sum of squared distances to the nearest centre BEFORE update i
 * (so entry iters is measured on the final centres). */
void ctkvr_oracle_kmeans(const float *X, int n, int dim, float *cent, int C, int iters, int is_bf16,
                         int32_t *assign_out, double *inertia_out)
{
    int64_t *sum = (int64_t *)malloc(sizeof(int64_t) * (size_t)C * dim);
    int32_t *cnt = (int32_t *)malloc(sizeof(int32_t) * (size_t)C);
    double *hn = (double *)malloc(sizeof(double) * (size_t)C);
    for (int it = 0; it <= iters; ++it) {
        for (int c = 0; c < C; ++c) {
            double a = 0.0;
            for (int e = 0; e < dim; ++e) a += (double)cent[(size_t)c * dim + e] * (double)cent[(size_t)c * dim + e];
            hn[c] = 0.5 * a;
        }
        double inertia = 0.0;
#pragma omp parallel for reduction(+ : inertia) schedule(static)
        for (int t = 0; t < n; ++t) {
            const float *x = X + (size_t)t * dim;
            double xx = 0.0;
            for (int e = 0; e < dim; ++e) xx += (double)x[e] * (double)x[e];
            double best = -INFINITY;
            int bi = 0;
            for (int c = 0; c < C; ++c) {
                const float *m = cent + (size_t)c * dim;
                double dot = 0.0;
                for (int e = 0; e < dim; ++e) dot += (double)x[e] * (double)m[e];
                double sc = dot - hn[c];          /* |x-m|^2 = |x|^2 - 2 (x.m - |m|^2/2) */
                if (sc > best) { best = sc; bi = c; }
            }
            assign_out[t] = bi;
            double d2 = xx - 2.0 * best;
            inertia += d2 > 0.0 ? d2 : 0.0;
        }
        inertia_out[it] = inertia;
        if (it == iters) break;
        memset(sum, 0, sizeof(int64_t) * (size_t)C * dim);
        memset(cnt, 0, sizeof(int32_t) * (size_t)C);
        for (int t = 0; t < n; ++t) {
            int c = assign_out[t];
            cnt[c] += 1;
            for (int e = 0; e < dim; ++e) sum[(size_t)c * dim + e] += (int64_t)llrint((double)X[(size_t)t * dim + e] * 1048576.0);
        }
        for (int c = 0; c < C; ++c) {
            if (cnt[c] == 0) continue;
            for (int e = 0; e < dim; ++e) {
                float m = (float)((double)sum[(size_t)c * dim + e] * (1.0 / 1048576.0) / (double)cnt[c]);
                cent[(size_t)c * dim + e] = is_bf16 ? round_bf16(m) : m;
            }
        }
    }
    free(sum);
    free(cnt);
    free(hn);
}
