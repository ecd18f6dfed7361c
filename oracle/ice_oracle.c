/*
 * CPU oracle for the IceCache hot path.  TEST INFRASTRUCTURE ONLY: nothing on the
 * product path may call, link or load this file; only the tests, the smoke check
 * and the benchmark's cpu_baseline leg do.  It shares no code with the HIP library.
 *
 * Plain, slow and meant to be checked against the paper by eye.  Every step is a
 * textbook definition written out:
 *   - nearest promoted point / nearest centroid = exhaustive argmin        (Sec. 4.2, Alg. 2)
 *   - centroid = arithmetic mean of the members                            (Lloyd step)
 *   - node -> pages: members in token order, cut every page_size tokens    (Sec. 4.1)       
 *   - insertion of a decode token under its nearest parent, on the raw
 *     keys or on the transformed ones                                      (Sec. 4.2, Alg. 1, Eq. 2)
 *   - page selection = full sort of all pages by score, take the first P   (Sec. 4.4, Alg. 3)
 *   - attention = masked softmax over the tokens of the selected pages     (Eq. 1)
 *
 * Arithmetic: inputs are bf16 bit patterns; dot products, norms, means and the
 * softmax are fp64.  Quantities that both sides must reproduce bit for bit are
 * defined in ordered fp32 (marked "ordered fp32" below): page sums, page
 * representatives, and the running cluster sums/means after an insertion.
 * Build with -ffp-contract=off so no fused multiply-add sneaks in.
 *
 * Pins (tests that tie this file to something other than itself) live in
 * tests/test_oracle_*.py: numpy brute force over the direct ||k-mu||^2 form,
 * a hand-written pagination example, sorted() for selection, dense softmax
 * attention when every page is selected, closed-form special cases.
 * Unpinned: none.
 *
 * All arrays carry a leading "unit" dimension: one unit = one (sequence, KV head)
 * pair, units are independent (Sec. 4.1: one tree per head).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t U, d, s, C, G, max_pages, max_tokens;
    int32_t *n_tokens;      /* [U] */
    int32_t *n_pages;       /* [U] */
    uint16_t *Kp, *Vp;      /* [U][max_pages][s][d] bf16 */
    int32_t *page_cluster;  /* [U][max_pages] */
    int32_t *page_fill;     /* [U][max_pages] */
    int32_t *page_pos;      /* [U][max_pages][s], -1 = empty slot */
    int32_t *cluster_tail;  /* [U][C] last page of the cluster, -1 = none */
    int32_t *cluster_cnt;   /* [U][C] */
    float *cluster_sum;     /* [U][C][d] */
    float *centroid;        /* [U][C][d] */
    float *page_sum;        /* [U][max_pages][d] */
    uint16_t *rep;          /* [U][max_pages][d] bf16 */
} orc_state_t;

static inline float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round to nearest, ties to even (finite inputs) */
static inline uint16_t f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int t) {
#ifdef _OPENMP
    omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* ---- nearest centroid: a_i = argmin_c ( w_c - 2 k_i . mu~_c ), w_c = ||mu~_c||^2 -------------
 * Exhaustive; lowest c wins ties.  mu~ is the bf16-rounded centroid.  (1-NN parent, Sec. 4.2.)
 * best/second receive the two smallest values of the objective per key (either may be NULL). */
void orc_assign(const uint16_t *K, const uint16_t *mu_bf16, int n, int C, int d,
                int32_t *a, double *best, double *second) {
    double *w = (double *)malloc(sizeof(double) * (size_t)C);
    for (int c = 0; c < C; ++c) {
        double acc = 0.0;
        for (int j = 0; j < d; ++j) {
            double m = bf16_to_f32(mu_bf16[(size_t)c * d + j]);
            acc += m * m;
        }
        w[c] = acc;
    }
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i) {
        double b1 = INFINITY, b2 = INFINITY;
        int arg = 0;
        for (int c = 0; c < C; ++c) {
            double dot = 0.0;
            for (int j = 0; j < d; ++j)
                dot += (double)bf16_to_f32(K[(size_t)i * d + j]) *
                       (double)bf16_to_f32(mu_bf16[(size_t)c * d + j]);
            double v = w[c] - 2.0 * dot;
            if (v < b1) { b2 = b1; b1 = v; arg = c; }
            else if (v < b2) { b2 = v; }
        }
        a[i] = arg;
        if (best) best[i] = b1;
        if (second) second[i] = b2;
    }
    free(w);
}

/* ---- centroid update: mean of the members; an empty cluster keeps its centroid -------------- */
void orc_means(const uint16_t *K, const int32_t *a, int n, int C, int d,
               float *mu, float *sum, int32_t *cnt) {
    double *acc = (double *)calloc((size_t)C * d, sizeof(double));
    for (int c = 0; c < C; ++c) cnt[c] = 0;
    for (int i = 0; i < n; ++i) {
        int c = a[i];
        cnt[c] += 1;
        for (int j = 0; j < d; ++j) acc[(size_t)c * d + j] += bf16_to_f32(K[(size_t)i * d + j]);
    }
    for (int c = 0; c < C; ++c)
        for (int j = 0; j < d; ++j) {
            sum[(size_t)c * d + j] = (float)acc[(size_t)c * d + j];
            if (cnt[c] > 0) mu[(size_t)c * d + j] = (float)(acc[(size_t)c * d + j] / cnt[c]);
        }
    free(acc);
}

/* ---- T Lloyd rounds from the promoted keys (one unit) ---------------------------------------
 * mu_c <- K[init_idx[c]]; each round: round mu to bf16, assign, recompute means.  The final
 * state is the last assignment and the means of that assignment.  inertia[t] (may be NULL) is
 * sum_i ||k_i - mu~_{a_i}||^2 seen by round t's assignment. */
void orc_lloyd(const uint16_t *K, int n, int C, int d, const int32_t *init_idx, int T,
               int32_t *a, float *mu, float *sum, int32_t *cnt, double *inertia) {
    uint16_t *mub = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)C * d);
    double *best = (double *)malloc(sizeof(double) * (size_t)n);
    for (int c = 0; c < C; ++c)
        for (int j = 0; j < d; ++j) mu[(size_t)c * d + j] = bf16_to_f32(K[(size_t)init_idx[c] * d + j]);
    for (int t = 0; t < T; ++t) {
        for (size_t x = 0; x < (size_t)C * d; ++x) mub[x] = f32_to_bf16(mu[x]);
        orc_assign(K, mub, n, C, d, a, best, NULL);
        if (inertia) {
            double tot = 0.0;
            for (int i = 0; i < n; ++i) {
                double kk = 0.0;
                for (int j = 0; j < d; ++j) {
                    double x = bf16_to_f32(K[(size_t)i * d + j]);
                    kk += x * x;
                }
                tot += best[i] + kk;
            }
            inertia[t] = tot;
        }
        orc_means(K, a, n, C, d, mu, sum, cnt);
    }
    free(mub);
    free(best);
}

/* page representative: ordered fp32 sum over the filled slots (slot 0 first, one add per slot,
 * no FMA), divided by the fill in fp32, rounded to bf16. */
static void page_rep(const orc_state_t *st, size_t u, int p) {
    const int d = st->d, s = st->s;
    const size_t pg = u * st->max_pages + p;
    const int fill = st->page_fill[pg];
    for (int j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int t = 0; t < fill; ++t) acc = acc + bf16_to_f32(st->Kp[(pg * s + t) * d + j]);
        st->page_sum[pg * d + j] = acc;
        st->rep[pg * d + j] = f32_to_bf16(acc / (float)fill);
    }
}

/* ---- node -> pages (one call = all units) ----------------------------------------------------
 * For c = 0..C-1 in order, members in ascending token position, cut every s tokens; page ids are
 * consecutive in that order.  K/V rows are bit copies.  Touches only the page tables, the page
 * pools, page sums and representatives, n_tokens and n_pages. */
void orc_paginate(orc_state_t *st, const uint16_t *K, const uint16_t *V, const int32_t *assign, int n) {
    const int d = st->d, s = st->s, C = st->C, MP = st->max_pages;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < st->U; ++u) {
        const uint16_t *Ku = K + (size_t)u * n * d, *Vu = V + (size_t)u * n * d;
        const int32_t *au = assign + (size_t)u * n;
        int np = 0;
        for (size_t x = 0; x < (size_t)MP; ++x) {
            st->page_cluster[(size_t)u * MP + x] = -1;
            st->page_fill[(size_t)u * MP + x] = 0;
        }
        for (size_t x = 0; x < (size_t)MP * s; ++x) st->page_pos[(size_t)u * MP * s + x] = -1;
        for (int c = 0; c < C; ++c) {
            int cur = -1;
            for (int i = 0; i < n; ++i) {
                if (au[i] != c) continue;
                if (cur < 0 || st->page_fill[(size_t)u * MP + cur] == s) {
                    cur = np++;
                    st->page_cluster[(size_t)u * MP + cur] = c;
                }
                size_t pg = (size_t)u * MP + cur;
                int slot = st->page_fill[pg]++;
                memcpy(st->Kp + (pg * s + slot) * d, Ku + (size_t)i * d, sizeof(uint16_t) * d);
                memcpy(st->Vp + (pg * s + slot) * d, Vu + (size_t)i * d, sizeof(uint16_t) * d);
                st->page_pos[pg * s + slot] = i;
            }
            st->cluster_tail[(size_t)u * C + c] = cur;
        }
        for (int p = 0; p < np; ++p) page_rep(st, (size_t)u, p);
        st->n_pages[u] = np;
        st->n_tokens[u] = n;
    }
}

/* ---- index build = Lloyd + paginate, all units ---------------------------------------------- */
void orc_build(orc_state_t *st, const uint16_t *K, const uint16_t *V, int n, const int32_t *init_idx,
               int T, int32_t *assign_out, double *inertia_out) {
    const int d = st->d, C = st->C;
    for (int u = 0; u < st->U; ++u)
        orc_lloyd(K + (size_t)u * n * d, n, C, d, init_idx + (size_t)u * C, T,
                  assign_out + (size_t)u * n, st->centroid + (size_t)u * C * d,
                  st->cluster_sum + (size_t)u * C * d, st->cluster_cnt + (size_t)u * C,
                  inertia_out ? inertia_out + (size_t)u * T : NULL);
    orc_paginate(st, K, V, assign_out, n);
}

/* ---- insertion of one decode token per unit ---------------------------------------------------
 * Nearest centroid as in orc_assign on the current bf16-rounded centroids; append to the
 * cluster's tail page (a fresh page if there is none or it is full); then, in ordered fp32:
 * page_sum += k, representative recomputed, cluster_sum += k, count+1, centroid = sum / count.
 * force[u] >= 0 overrides the argmin (used to follow the other side through a near-tie).
 * chosen/best/second report the decision and the two smallest objective values.
 * Returns 0, or -1 if a unit is out of token capacity (nothing is modified then).  Pages cannot
 * run out: max_pages = floor(max_tokens / s) + C covers every full page plus one partial page
 * per cluster.
 *
 * With a geometry (orc_insert_transformed) the distances are those between TRANSFORMED keys
 * (Sec. 4.2 last paragraph: a decode token is inserted under its nearest parent in the same space
 * the tree was built in; Eq. 2: T_K(k) = [k / c, sqrt(1 - ||k||^2 / c^2)]).  Kept times c, a key is
 * the row [k, a(k)] with ONE more coordinate a(k) = sqrt(c^2 - ||k||^2), rounded to bf16 like every
 * stored coordinate; a key beyond the radius (||k|| > c, which Eq. 2 does not cover: c was fixed at
 * prefill) gets a = 0.  Centroids carry the mean of their members' a.  Everything is the raw
 * insertion on (d+1)-dimensional rows: the argmin runs over w_c - 2 [k,a].[mu~_c, e~_c] with
 * w_c = ||mu~_c||^2 + e~_c^2 (e~ = the extra coordinate of the centroid rounded to bf16), and the
 * extra coordinate's running sum and mean move in ordered fp32 exactly like the other d.
 * Page tiles, page sums and representatives hold the d raw coordinates only (the transformed query
 * has 0 in the extra one, Eq. 3).  extra_override[u] >= 0 replaces the oracle's own a(k) bits (to
 * follow the other side when its fp32 norm lands on the other side of a bf16 rounding boundary);
 * extra_out reports the oracle's own. */
typedef struct {
    float *radius_sq;          /* [U] c^2, fixed at prefill */
    uint16_t *key_extra;       /* [U][max_tokens] bf16 a(k) by token position */
    float *centroid_extra;     /* [U][C] mean of the members' a */
    float *cluster_sum_extra;  /* [U][C] their running sum */
} orc_geometry_t;

static void insert_one(orc_state_t *st, orc_geometry_t *geo, int u, const uint16_t *ku, const uint16_t *vu,
                       const int32_t *force, const int32_t *extra_override, int32_t *chosen, double *best,
                       double *second, uint16_t *extra_out) {
    const int d = st->d, s = st->s, C = st->C, MP = st->max_pages;
    /* the new key's extra coordinate (transformed geometry only) */
    uint16_t a_bits = 0;
    double a_val = 0.0;
    if (geo) {
        double n2 = 0.0;
        for (int j = 0; j < d; ++j) {
            double x = bf16_to_f32(ku[j]);
            n2 += x * x;
        }
        double rest = (double)geo->radius_sq[u] - n2;
        a_bits = f32_to_bf16((float)sqrt(rest > 0.0 ? rest : 0.0));   /* beyond the radius: 0 */
        if (extra_out) extra_out[u] = a_bits;
        if (extra_override && extra_override[u] >= 0) a_bits = (uint16_t)extra_override[u];
        a_val = bf16_to_f32(a_bits);
    }
    /* exhaustive search over the bf16-rounded centroids, as orc_assign does for one key */
    int32_t arg = 0;
    double b1 = INFINITY, b2 = INFINITY;
    for (int c = 0; c < C; ++c) {
        double w = 0.0, dot = 0.0;
        for (int j = 0; j < d; ++j) {
            double m = bf16_to_f32(f32_to_bf16(st->centroid[((size_t)u * C + c) * d + j]));
            w += m * m;
            dot += (double)bf16_to_f32(ku[j]) * m;
        }
        if (geo) {
            double e = bf16_to_f32(f32_to_bf16(geo->centroid_extra[(size_t)u * C + c]));
            w += e * e;
            dot += a_val * e;
        }
        double val = w - 2.0 * dot;
        if (val < b1) { b2 = b1; b1 = val; arg = c; }
        else if (val < b2) { b2 = val; }
    }
    if (force && force[u] >= 0) arg = force[u];
    if (chosen) chosen[u] = arg;
    if (best) best[u] = b1;
    if (second) second[u] = b2;

    int tail = st->cluster_tail[(size_t)u * C + arg];
    if (tail < 0 || st->page_fill[(size_t)u * MP + tail] == s) {
        tail = st->n_pages[u]++;
        st->cluster_tail[(size_t)u * C + arg] = tail;
        st->page_cluster[(size_t)u * MP + tail] = arg;
        st->page_fill[(size_t)u * MP + tail] = 0;
        for (int j = 0; j < d; ++j) st->page_sum[((size_t)u * MP + tail) * d + j] = 0.0f;
    }
    size_t pg = (size_t)u * MP + tail;
    int slot = st->page_fill[pg]++;
    memcpy(st->Kp + (pg * s + slot) * d, ku, sizeof(uint16_t) * d);
    memcpy(st->Vp + (pg * s + slot) * d, vu, sizeof(uint16_t) * d);
    const int tok = st->n_tokens[u]++;
    st->page_pos[pg * s + slot] = tok;
    int fill = slot + 1;
    size_t cl = (size_t)u * C + arg;
    int cnt = ++st->cluster_cnt[cl];
    for (int j = 0; j < d; ++j) {
        float kf = bf16_to_f32(ku[j]);
        float ps = st->page_sum[pg * d + j] + kf;             /* ordered fp32 */
        st->page_sum[pg * d + j] = ps;
        st->rep[pg * d + j] = f32_to_bf16(ps / (float)fill);
        float cs = st->cluster_sum[cl * d + j] + kf;          /* ordered fp32 */
        st->cluster_sum[cl * d + j] = cs;
        st->centroid[cl * d + j] = cs / (float)cnt;
    }
    if (geo) {
        float es = geo->cluster_sum_extra[cl] + bf16_to_f32(a_bits);   /* ordered fp32 */
        geo->cluster_sum_extra[cl] = es;
        geo->centroid_extra[cl] = es / (float)cnt;
        geo->key_extra[(size_t)u * st->max_tokens + tok] = a_bits;
    }
}

int orc_insert(orc_state_t *st, const uint16_t *k, const uint16_t *v, const int32_t *force,
               int32_t *chosen, double *best, double *second) {
    const int d = st->d;
    for (int u = 0; u < st->U; ++u)
        if (st->n_tokens[u] >= st->max_tokens) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < st->U; ++u)
        insert_one(st, NULL, u, k + (size_t)u * d, v + (size_t)u * d, force, NULL, chosen, best, second, NULL);
    return 0;
}

int orc_insert_transformed(orc_state_t *st, orc_geometry_t *geo, const uint16_t *k, const uint16_t *v,
                           const int32_t *force, const int32_t *extra_override, int32_t *chosen, double *best,
                           double *second, uint16_t *extra_out) {
    const int d = st->d;
    for (int u = 0; u < st->U; ++u)
        if (st->n_tokens[u] >= st->max_tokens) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < st->U; ++u)
        insert_one(st, geo, u, k + (size_t)u * d, v + (size_t)u * d, force, extra_override, chosen, best, second,
                   extra_out);
    return 0;
}

/* ---- page selection ---------------------------------------------------------------------------
 * P = floor(budget / s) pages per unit; n_sel = min(P, n_pages).  Score of page p for query head
 * h: (q_h . rep_p) / ||q_h||  (the query normalisation T_Q, Eq. 3); group score = max over
 * the G heads that share the KV head (GQA sharing, Sec. 4.3).  Scores are computed in fp64 and
 * rounded once to fp32, the precision the decision is taken in.  Full sort of ALL pages by
 * (score descending, page id ascending); the first n_sel are returned with ids ascending,
 * padded with -1.  scores[] (may be NULL) = group scores of the returned ids; S_all (may be
 * NULL, [U][max_pages]) = every page's fp32 group score. */
typedef struct { float s; int32_t id; } scored_t;

static int cmp_scored(const void *a, const void *b) {
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

static int cmp_i32(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

void orc_select(const orc_state_t *st, const uint16_t *q, int budget, int32_t *ids, int32_t *n_sel,
                float *scores, float *S_all) {
    const int d = st->d, G = st->G, MP = st->max_pages, P = budget / st->s;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < st->U; ++u) {
        const int np = st->n_pages[u];
        scored_t *sc = (scored_t *)malloc(sizeof(scored_t) * (size_t)(np > 0 ? np : 1));
        double qn[64];
        for (int h = 0; h < G; ++h) {
            double acc = 0.0;
            for (int j = 0; j < d; ++j) {
                double x = bf16_to_f32(q[((size_t)u * G + h) * d + j]);
                acc += x * x;
            }
            qn[h] = sqrt(acc);
            if (qn[h] < 1e-20) qn[h] = 1e-20;
        }
        for (int p = 0; p < np; ++p) {
            double best = -INFINITY;
            for (int h = 0; h < G; ++h) {
                double dot = 0.0;
                for (int j = 0; j < d; ++j)
                    dot += (double)bf16_to_f32(q[((size_t)u * G + h) * d + j]) *
                           (double)bf16_to_f32(st->rep[((size_t)u * MP + p) * d + j]);
                double sh = dot / qn[h];
                if (sh > best) best = sh;
            }
            sc[p].s = (float)best;
            sc[p].id = p;
            if (S_all) S_all[(size_t)u * MP + p] = (float)best;
        }
        qsort(sc, (size_t)np, sizeof(scored_t), cmp_scored);
        int ns = np < P ? np : P;
        int32_t *out = ids + (size_t)u * P;
        for (int x = 0; x < ns; ++x) out[x] = sc[x].id;
        qsort(out, (size_t)ns, sizeof(int32_t), cmp_i32);
        for (int x = ns; x < P; ++x) out[x] = -1;
        if (scores) {
            for (int x = 0; x < P; ++x) scores[(size_t)u * P + x] = 0.0f;
            for (int x = 0; x < ns; ++x)
                for (int y = 0; y < ns; ++y)
                    if (sc[y].id == out[x]) scores[(size_t)u * P + x] = sc[y].s;
        }
        n_sel[u] = ns;
        free(sc);
    }
}

/* ---- hierarchical page selection ----------------------------------------------------------------
 * The two-level form of the paper's top-down search (Sec. 3.3, Alg. 4: level by level, descend
 * from the parents that score best to their children; page selection, Alg. 3, calls it).
 * Stage 1 scores the C cluster centroids, rounded to bf16 as the index stores them, with the same normalised GQA score as the pages (max over the
 * group's heads of q_h . mu~_c / ||q_h||, fp64 rounded once to fp32) and keeps the
 * n_keep = min(n_probe, C) best by (score descending, cluster id ascending); every cluster is
 * eligible, one without pages simply contributes none.  Stage 2 ranks only the live pages whose
 * cluster was kept, exactly as orc_select ranks all pages, and returns the best
 * min(P, number of such pages), ids ascending, padded with -1.  With n_probe >= C every page is
 * a candidate and the result is orc_select's.
 * Stage 3 (n_refine > 0; the paper ranks KEYS and then loads the pages that hold them, Alg. 3):
 * only the min(n_refine, candidates) best pages of stage 2 stay; each is re-scored by its best
 * key, max over its tokens and the group's heads of q_h . k / ||q_h|| (fp64 rounded once to
 * fp32), and the best min(P, kept) by (that score descending, page id ascending) are returned;
 * scores[] then holds these key scores.
 * clusters (may be NULL): [U][n_probe] kept cluster ids ascending, -1 padded.
 * Sc_all (may be NULL): [U][C] fp32 centroid scores. */
static void select_hier_impl(const orc_state_t *st, const uint16_t *q, int budget, int n_probe, int n_refine,
                             const char *eligible /* [U][C] or NULL: clusters that may be kept */, int32_t *ids,
                             int32_t *n_sel, float *scores, int32_t *clusters, float *Sc_all) {
    const int d = st->d, G = st->G, MP = st->max_pages, C = st->C, P = budget / st->s;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < st->U; ++u) {
        const int np = st->n_pages[u];
        double qn[64];
        for (int h = 0; h < G; ++h) {
            double acc = 0.0;
            for (int j = 0; j < d; ++j) {
                double x = bf16_to_f32(q[((size_t)u * G + h) * d + j]);
                acc += x * x;
            }
            qn[h] = sqrt(acc);
            if (qn[h] < 1e-20) qn[h] = 1e-20;
        }
        /* stage 1: clusters */
        scored_t *cs = (scored_t *)malloc(sizeof(scored_t) * (size_t)C);
        for (int c = 0; c < C; ++c) {
            double best = -INFINITY;
            for (int h = 0; h < G; ++h) {
                double dot = 0.0;
                for (int j = 0; j < d; ++j) {
                    float mu = bf16_to_f32(f32_to_bf16(st->centroid[((size_t)u * C + c) * d + j]));
                    dot += (double)bf16_to_f32(q[((size_t)u * G + h) * d + j]) * (double)mu;
                }
                double sh = dot / qn[h];
                if (sh > best) best = sh;
            }
            cs[c].s = (float)best;
            cs[c].id = c;
            if (Sc_all) Sc_all[(size_t)u * C + c] = (float)best;
        }
        /* the eligible clusters first (all of them without a level above), best first */
        int n_el = 0;
        for (int c = 0; c < C; ++c)
            if (!eligible || eligible[(size_t)u * C + c]) cs[n_el++] = cs[c];
        qsort(cs, (size_t)n_el, sizeof(scored_t), cmp_scored);
        const int n_keep = n_probe < n_el ? n_probe : n_el;
        char *kept = (char *)calloc((size_t)C, 1);
        for (int x = 0; x < n_keep; ++x) kept[cs[x].id] = 1;
        if (clusters) {
            int w = 0;
            for (int c = 0; c < C; ++c)
                if (kept[c]) clusters[(size_t)u * n_probe + w++] = c;
            for (; w < n_probe; ++w) clusters[(size_t)u * n_probe + w] = -1;
        }
        /* stage 2: the pages of the kept clusters */
        scored_t *sc = (scored_t *)malloc(sizeof(scored_t) * (size_t)(np > 0 ? np : 1));
        int nc = 0;
        for (int p = 0; p < np; ++p) {
            const int c = st->page_cluster[(size_t)u * MP + p];
            if (c < 0 || c >= C || !kept[c]) continue;
            double best = -INFINITY;
            for (int h = 0; h < G; ++h) {
                double dot = 0.0;
                for (int j = 0; j < d; ++j)
                    dot += (double)bf16_to_f32(q[((size_t)u * G + h) * d + j]) *
                           (double)bf16_to_f32(st->rep[((size_t)u * MP + p) * d + j]);
                double sh = dot / qn[h];
                if (sh > best) best = sh;
            }
            sc[nc].s = (float)best;
            sc[nc].id = p;
            ++nc;
        }
        qsort(sc, (size_t)nc, sizeof(scored_t), cmp_scored);
        if (n_refine > 0) {
            /* stage 3: the best pages by representative, re-scored by their best key */
            if (nc > n_refine) nc = n_refine;
            for (int x = 0; x < nc; ++x) {
                const size_t pg = (size_t)u * MP + sc[x].id;
                double best = -INFINITY;
                for (int t = 0; t < st->page_fill[pg]; ++t)
                    for (int h = 0; h < G; ++h) {
                        double dot = 0.0;
                        for (int j = 0; j < d; ++j)
                            dot += (double)bf16_to_f32(q[((size_t)u * G + h) * d + j]) *
                                   (double)bf16_to_f32(st->Kp[(pg * st->s + t) * d + j]);
                        double sh = dot / qn[h];
                        if (sh > best) best = sh;
                    }
                sc[x].s = (float)best;
            }
            qsort(sc, (size_t)nc, sizeof(scored_t), cmp_scored);
        }
        int ns = nc < P ? nc : P;
        int32_t *out = ids + (size_t)u * P;
        for (int x = 0; x < ns; ++x) out[x] = sc[x].id;
        qsort(out, (size_t)ns, sizeof(int32_t), cmp_i32);
        for (int x = ns; x < P; ++x) out[x] = -1;
        if (scores) {
            for (int x = 0; x < P; ++x) scores[(size_t)u * P + x] = 0.0f;
            for (int x = 0; x < ns; ++x)
                for (int y = 0; y < ns; ++y)
                    if (sc[y].id == out[x]) scores[(size_t)u * P + x] = sc[y].s;
        }
        n_sel[u] = ns;
        free(sc);
        free(kept);
        free(cs);
    }
}

void orc_select_hier(const orc_state_t *st, const uint16_t *q, int budget, int n_probe, int n_refine, int32_t *ids,
                     int32_t *n_sel, float *scores, int32_t *clusters, float *Sc_all) {
    select_hier_impl(st, q, budget, n_probe, n_refine, NULL, ids, n_sel, scores, clusters, Sc_all);
}

/* ---- three levels ---------------------------------------------------------------------------------
 * One more level of the tree above the clusters (Sec. 3.3: levels L..1, every point's parent is a
 * point of the level above; Alg. 4 descends from the top level, keeping the best nodes of a level
 * and searching only their children on the next).  The top level is given as state: top_centroid
 * fp32 [U][C2][d] (a top node's position) and top_of int32 [U][C] (the top node each cluster
 * hangs under).  Stage 0 scores the C2 top nodes, rounded to bf16, with the same normalised GQA
 * score as everything below (max over the group's heads of q_h . t / ||q_h||, fp64 rounded once to
 * fp32) and keeps the min(n_probe_top, C2) best by (score descending, id ascending).  Stage 1 is
 * orc_select_hier's, restricted to the clusters whose top node was kept (the best
 * min(n_probe, number of such clusters) of them); stages 2 and 3 follow unchanged.  With
 * n_probe_top >= C2 every cluster is eligible and the result is orc_select_hier's.
 * tops (may be NULL): [U][n_probe_top] kept top nodes ascending, -1 padded; St_all (may be NULL):
 * [U][C2] fp32 top-node scores. */
void orc_select_hier3(const orc_state_t *st, const float *top_centroid, const int32_t *top_of, int C2,
                      const uint16_t *q, int budget, int n_probe_top, int n_probe, int n_refine, int32_t *ids,
                      int32_t *n_sel, float *scores, int32_t *clusters, int32_t *tops, float *Sc_all, float *St_all) {
    const int d = st->d, G = st->G, C = st->C;
    const int n_keep0 = n_probe_top < C2 ? n_probe_top : C2;
    char *eligible = (char *)calloc((size_t)st->U * C, 1);
    for (int u = 0; u < st->U; ++u) {
        double qn[64];
        for (int h = 0; h < G; ++h) {
            double acc = 0.0;
            for (int j = 0; j < d; ++j) {
                double x = bf16_to_f32(q[((size_t)u * G + h) * d + j]);
                acc += x * x;
            }
            qn[h] = sqrt(acc);
            if (qn[h] < 1e-20) qn[h] = 1e-20;
        }
        scored_t *ts = (scored_t *)malloc(sizeof(scored_t) * (size_t)C2);
        for (int t = 0; t < C2; ++t) {
            double best = -INFINITY;
            for (int h = 0; h < G; ++h) {
                double dot = 0.0;
                for (int j = 0; j < d; ++j) {
                    float tc = bf16_to_f32(f32_to_bf16(top_centroid[((size_t)u * C2 + t) * d + j]));
                    dot += (double)bf16_to_f32(q[((size_t)u * G + h) * d + j]) * (double)tc;
                }
                double sh = dot / qn[h];
                if (sh > best) best = sh;
            }
            ts[t].s = (float)best;
            ts[t].id = t;
            if (St_all) St_all[(size_t)u * C2 + t] = (float)best;
        }
        qsort(ts, (size_t)C2, sizeof(scored_t), cmp_scored);
        char *kept0 = (char *)calloc((size_t)C2, 1);
        for (int x = 0; x < n_keep0; ++x) kept0[ts[x].id] = 1;
        if (tops) {
            int w = 0;
            for (int t = 0; t < C2; ++t)
                if (kept0[t]) tops[(size_t)u * n_probe_top + w++] = t;
            for (; w < n_probe_top; ++w) tops[(size_t)u * n_probe_top + w] = -1;
        }
        for (int c = 0; c < C; ++c) {
            const int t = top_of[(size_t)u * C + c];
            eligible[(size_t)u * C + c] = (t >= 0 && t < C2 && kept0[t]) ? 1 : 0;
        }
        free(kept0);
        free(ts);
    }
    select_hier_impl(st, q, budget, n_probe, n_refine, eligible, ids, n_sel, scores, clusters, Sc_all);
    free(eligible);
}

/* ---- sparse attention over the selected pages (Eq. 1 with the mask = selected tokens) ---------
 * For every query head of the group: logits z = q.k / sqrt(d) over every filled slot of every
 * selected page, softmax with the maximum subtracted, output = sum softmax * v.  fp64, output
 * rounded to fp32.  No selected token -> zeros.  ids: [U][P], first n_sel[u] entries used. */
void orc_attend(const orc_state_t *st, const uint16_t *q, const int32_t *ids, const int32_t *n_sel,
                int P, float *out) {
    const int d = st->d, s = st->s, G = st->G, MP = st->max_pages;
    const double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < st->U; ++u) {
        const int ns = n_sel[u];
        double *z = (double *)malloc(sizeof(double) * (size_t)(ns > 0 ? ns : 1) * s);
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
        for (int h = 0; h < G; ++h) {
            const uint16_t *qh = q + ((size_t)u * G + h) * d;
            int m = 0;
            double zmax = -INFINITY;
            for (int x = 0; x < ns; ++x) {
                size_t pg = (size_t)u * MP + ids[(size_t)u * P + x];
                for (int t = 0; t < st->page_fill[pg]; ++t) {
                    double dot = 0.0;
                    for (int j = 0; j < d; ++j)
                        dot += (double)bf16_to_f32(qh[j]) * (double)bf16_to_f32(st->Kp[(pg * s + t) * d + j]);
                    z[m] = dot * scale;
                    if (z[m] > zmax) zmax = z[m];
                    ++m;
                }
            }
            double den = 0.0;
            for (int j = 0; j < d; ++j) o[j] = 0.0;
            m = 0;
            for (int x = 0; x < ns; ++x) {
                size_t pg = (size_t)u * MP + ids[(size_t)u * P + x];
                for (int t = 0; t < st->page_fill[pg]; ++t) {
                    double e = exp(z[m++] - zmax);
                    den += e;
                    for (int j = 0; j < d; ++j) o[j] += e * (double)bf16_to_f32(st->Vp[(pg * s + t) * d + j]);
                }
            }
            float *oh = out + ((size_t)u * G + h) * d;
            for (int j = 0; j < d; ++j) oh[j] = (m > 0) ? (float)(o[j] / den) : 0.0f;
        }
        free(z);
        free(o);
    }
}

/* ---- sparse attention with resident tokens -----------------------------------------------------
 * The decode loop of the paper (Alg. 1, App. A) always attends to the sink tokens at the start of
 * the sequence and to a window of the most recent tokens, which are not (yet) in the index; the
 * selected pages come on top.  Here the resident tokens are one dense run per unit:
 * rk, rv bf16 [U][n_res][d].  One softmax over the tokens of the listed pages and the resident
 * tokens together (Eq. 1 with the mask on their union). */
void orc_attend_resident(const orc_state_t *st, const uint16_t *q, const int32_t *ids, const int32_t *n_sel,
                         int P, const uint16_t *rk, const uint16_t *rv, int n_res, float *out) {
    const int d = st->d, s = st->s, G = st->G, MP = st->max_pages;
    const double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < st->U; ++u) {
        const int ns = n_sel[u];
        /* rows of every attended token, in any order */
        size_t cap = (size_t)(ns > 0 ? ns : 0) * s + (size_t)n_res + 1;
        const uint16_t **kr = (const uint16_t **)malloc(sizeof(void *) * cap);
        const uint16_t **vr = (const uint16_t **)malloc(sizeof(void *) * cap);
        int m = 0;
        for (int x = 0; x < ns; ++x) {
            size_t pg = (size_t)u * MP + ids[(size_t)u * P + x];
            for (int t = 0; t < st->page_fill[pg]; ++t) {
                kr[m] = st->Kp + (pg * s + t) * d;
                vr[m] = st->Vp + (pg * s + t) * d;
                ++m;
            }
        }
        for (int t = 0; t < n_res; ++t) {
            kr[m] = rk + ((size_t)u * n_res + t) * d;
            vr[m] = rv + ((size_t)u * n_res + t) * d;
            ++m;
        }
        double *z = (double *)malloc(sizeof(double) * (size_t)(m > 0 ? m : 1));
        for (int h = 0; h < G; ++h) {
            const uint16_t *qh = q + ((size_t)u * G + h) * d;
            double zmax = -INFINITY;
            for (int i = 0; i < m; ++i) {
                double dot = 0.0;
                for (int j = 0; j < d; ++j) dot += (double)bf16_to_f32(qh[j]) * (double)bf16_to_f32(kr[i][j]);
                z[i] = dot * scale;
                if (z[i] > zmax) zmax = z[i];
            }
            double den = 0.0;
            for (int i = 0; i < m; ++i) {
                z[i] = exp(z[i] - zmax);
                den += z[i];
            }
            float *oh = out + ((size_t)u * G + h) * d;
            for (int j = 0; j < d; ++j) {
                double o = 0.0;
                for (int i = 0; i < m; ++i) o += z[i] * (double)bf16_to_f32(vr[i][j]);
                oh[j] = (m > 0) ? (float)(o / den) : 0.0f;
            }
        }
        free(z);
        free(kr);
        free(vr);
    }
}

/* ---- reuse of a selection by other layers (App. B) ---------------------------------------------
 * Page ids are local to one layer's index; the sequence positions of the tokens in those pages
 * are not.  orc_selected_tokens lists them (list order, then slot order; -1 padded to P * s);
 * orc_attend_tokens attends over rows pos[u][0 .. n_tok[u]) of a dense cache K, V [U][n_rows][d]:
 * one softmax over exactly those rows (Eq. 1 with the mask on them). */
void orc_selected_tokens(const orc_state_t *st, const int32_t *ids, const int32_t *n_sel, int P,
                         int32_t *pos, int32_t *n_tok) {
    const int s = st->s, MP = st->max_pages;
    for (int u = 0; u < st->U; ++u) {
        int m = 0;
        for (int x = 0; x < n_sel[u]; ++x) {
            size_t pg = (size_t)u * MP + ids[(size_t)u * P + x];
            for (int t = 0; t < st->page_fill[pg]; ++t) pos[(size_t)u * P * s + m++] = st->page_pos[pg * s + t];
        }
        n_tok[u] = m;
        for (; m < P * s; ++m) pos[(size_t)u * P * s + m] = -1;
    }
}

void orc_attend_tokens(const uint16_t *q, const uint16_t *K, const uint16_t *V, int U, int G, int d, int n_rows,
                       const int32_t *pos, const int32_t *n_tok, int cap, float *out) {
    const double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < U; ++u) {
        const int m = n_tok[u];
        double *z = (double *)malloc(sizeof(double) * (size_t)(m > 0 ? m : 1));
        for (int h = 0; h < G; ++h) {
            const uint16_t *qh = q + ((size_t)u * G + h) * d;
            double zmax = -INFINITY;
            for (int i = 0; i < m; ++i) {
                const uint16_t *kr = K + ((size_t)u * n_rows + pos[(size_t)u * cap + i]) * d;
                double dot = 0.0;
                for (int j = 0; j < d; ++j) dot += (double)bf16_to_f32(qh[j]) * (double)bf16_to_f32(kr[j]);
                z[i] = dot * scale;
                if (z[i] > zmax) zmax = z[i];
            }
            double den = 0.0;
            for (int i = 0; i < m; ++i) {
                z[i] = exp(z[i] - zmax);
                den += z[i];
            }
            float *oh = out + ((size_t)u * G + h) * d;
            for (int j = 0; j < d; ++j) {
                double o = 0.0;
                for (int i = 0; i < m; ++i)
                    o += z[i] * (double)bf16_to_f32(V[((size_t)u * n_rows + pos[(size_t)u * cap + i]) * d + j]);
                oh[j] = (m > 0) ? (float)(o / den) : 0.0f;
            }
        }
        free(z);
    }
}
