/*
 * CPU oracle of one LoLA attention layer (arxiv 2505.23666).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the layer
 * computes, written from the paper's definitions.  It shares no code with the HIP library and
 * must never be called from the product path; only tests, the smoke check and the benchmark's
 * CPU-baseline leg load it.
 *
 * Arithmetic: every quantity is held in `real` (double unless ORC_REAL is overridden at compile
 * time; a float build exists only to show how far plain fp32 arithmetic drifts from fp64).
 * Inputs arrive as float arrays that already hold values representable in the mode's storage
 * type (bf16 or fp32), so the conversion to `real` is exact and nothing is rounded in between.
 *
 * What follows the paper, passage by passage:
 *   phi_map            - feature map, Sec. 2.3 eq. (feature_map); the SOFTMAX kind is the bounded
 *                        variant the benchmark configurations prescribe: [softmax(z), softmax(-z)]
 *   sre                - self-recall error, Sec. 3 eq. (score)
 *   fold_pair          - recurrent update, Sec. 2.2 eq. (recurrent_update) / Sec. 3 (H_t, s_t update)
 *   select_and_fold    - top-lambda of the eligible set, rest folded, Sec. 3 (G_t argmax, S_t)
 *   attend             - output under the shared normaliser, Sec. 3 (y_t equation)
 *   orc_decode_step    - generation-time order: update caches, then attend (Sec. 3, text before the
 *                        y_t equation; appendix "Algorithm Pseudo-Code", update/attend)
 *   orc_prefill        - chunkwise inference, Sec. 3 "Chunkwise Inference" (E_t for chunks) and
 *                        appendix update_chunk
 *   orc_cache_elems    - cache-size accounting, appendix "LoLA Cache vs. Transformers"
 *   cfg.score_kind     - the alternative, query-dependent importance scores of Sec. 4 "scoring ablation"
 *                        / appendix "scoring ablation": Score(k_i) = sum over the eta queries
 *                        t = i .. i+eta-1 that see k_i in the sliding window (all query heads of the
 *                        group) of (w - a)^2, |w - a|, a / w or w, with w = exp(scale q_t.k_i) and
 *                        a = phi(q_t).phi(k_i); the score is final when the pair leaves the window
 *                        and is kept with it in the sparse cache (query_term, accumulate_scores)
 *   cfg.hide           - restricted-query ablation, appendix "Sparse Cache & Linear Attention
 *                        Ablation": the memories are updated as usual, but the query does not read
 *                        the hidden state (bit 0) and / or the sparse cache (bit 1)
 *
 * Readings taken where the paper is silent or ambiguous (each is also listed in the design notes):
 *   - scoring uses the state *before* the update of the same step (both pseudo-codes do);
 *   - recall := 0 while nothing has been folded (phi(k)^T s = 0), so SRE = ||v||;
 *   - while |E| <= lambda everything is kept and nothing is scored or folded;
 *   - exactly lambda pairs are kept; order is (SRE descending, token index ascending);
 *   - a folded pair never returns;
 *   - GQA: state, caches, scoring and selection live per kv head; query head hq reads kv head
 *     hq / (Hq/Hkv);
 *   - prefill keeps the boundary invariant "window = last min(n, eta) tokens": after the outputs
 *     of a chunk, window ++ chunk is cut to its last eta tokens and the cut-off prefix is the
 *     evicted group of that chunk (one selection for the whole group).
 * No max-subtraction is applied to the exponentials: logits are assumed to stay far below the
 * overflow threshold of `real` (true for every workload this oracle is used on).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef ORC_REAL
#define ORC_REAL double
#endif
typedef ORC_REAL real;

enum { ORC_PHI_SOFTMAX = 0, ORC_PHI_EXP = 1 };
enum { ORC_SCORE_SRE = 0, ORC_SCORE_WERR_SQ = 1, ORC_SCORE_WERR_ABS = 2, ORC_SCORE_OVEREST = 3, ORC_SCORE_ATTN = 4 };

typedef struct {
    int32_t B, Hq, Hkv, d, D, eta, lambda, C, phi_kind;
    double scale; /* logit scale; <= 0 means 1/sqrt(d) */
    int32_t hide; /* bit 0: queries do not read (H, s); bit 1: queries do not read the sparse cache */
    int32_t score_kind; /* ORC_SCORE_*: what ranks the eligible pairs */
} orc_config;

typedef struct {
    real *k, *v;   /* [cap][d] */
    int64_t *idx;  /* [cap] token index */
    real *score;   /* [cap] query-dependent score gathered so far (unused with ORC_SCORE_SRE) */
    int n, cap;
} pair_list;

typedef struct {
    real *H; /* [D][d] */
    real *s; /* [D] */
    pair_list win; /* chronological, win.k[0] is the oldest */
    pair_list sp;  /* sparse cache, unordered */
    int64_t *folded; int64_t n_folded, cap_folded;
    int64_t n_scored_events, n_adopted, n_mismatch;
    double min_margin;
} stream_t;

typedef struct {
    orc_config cfg;
    stream_t *st;       /* [B*Hkv] */
    int64_t *n_tokens;  /* [B] */
} orc_state;

/* ------------------------------------------------------------------------------------------ */

static void pl_init(pair_list *p, int cap, int d) {
    p->cap = cap > 0 ? cap : 1;
    p->k = (real *)calloc((size_t)p->cap * d, sizeof(real));
    p->v = (real *)calloc((size_t)p->cap * d, sizeof(real));
    p->idx = (int64_t *)calloc((size_t)p->cap, sizeof(int64_t));
    p->score = (real *)calloc((size_t)p->cap, sizeof(real));
    p->n = 0;
}
static void pl_free(pair_list *p) { free(p->k); free(p->v); free(p->idx); free(p->score); }
static void pl_reserve(pair_list *p, int cap, int d) {
    if (cap <= p->cap) return;
    p->k = (real *)realloc(p->k, (size_t)cap * d * sizeof(real));
    p->v = (real *)realloc(p->v, (size_t)cap * d * sizeof(real));
    p->idx = (int64_t *)realloc(p->idx, (size_t)cap * sizeof(int64_t));
    p->score = (real *)realloc(p->score, (size_t)cap * sizeof(real));
    p->cap = cap;
}
static void pl_push_scored(pair_list *p, int d, const real *k, const real *v, int64_t idx, real score) {
    if (p->n == p->cap) pl_reserve(p, 2 * p->cap, d);
    memcpy(p->k + (size_t)p->n * d, k, d * sizeof(real));
    memcpy(p->v + (size_t)p->n * d, v, d * sizeof(real));
    p->idx[p->n] = idx;
    p->score[p->n] = score;
    p->n++;
}
static void pl_push(pair_list *p, int d, const real *k, const real *v, int64_t idx) { pl_push_scored(p, d, k, v, idx, 0); }
/* drop the first `cnt` entries */
static void pl_drop_front(pair_list *p, int d, int cnt) {
    int rest = p->n - cnt;
    memmove(p->k, p->k + (size_t)cnt * d, (size_t)rest * d * sizeof(real));
    memmove(p->v, p->v + (size_t)cnt * d, (size_t)rest * d * sizeof(real));
    memmove(p->idx, p->idx + cnt, (size_t)rest * sizeof(int64_t));
    memmove(p->score, p->score + cnt, (size_t)rest * sizeof(real));
    p->n = rest;
}

orc_state *orc_state_new(const orc_config *cfg) {
    if (!cfg || cfg->B < 1 || cfg->Hkv < 1 || cfg->Hq < cfg->Hkv || cfg->Hq % cfg->Hkv ||
        cfg->d < 1 || cfg->D < 2 || (cfg->D & 1) || cfg->eta < 0 || cfg->lambda < 0 || cfg->C < 1)
        return NULL;
    orc_state *S = (orc_state *)calloc(1, sizeof(orc_state));
    S->cfg = *cfg;
    if (S->cfg.scale <= 0) S->cfg.scale = 1.0 / sqrt((double)cfg->d);
    int ns = cfg->B * cfg->Hkv;
    S->st = (stream_t *)calloc((size_t)ns, sizeof(stream_t));
    S->n_tokens = (int64_t *)calloc((size_t)cfg->B, sizeof(int64_t));
    for (int i = 0; i < ns; i++) {
        stream_t *t = &S->st[i];
        t->H = (real *)calloc((size_t)cfg->D * cfg->d, sizeof(real));
        t->s = (real *)calloc((size_t)cfg->D, sizeof(real));
        pl_init(&t->win, cfg->eta + cfg->C + 1, cfg->d);
        pl_init(&t->sp, cfg->lambda + cfg->C + cfg->eta + 1, cfg->d);
        t->cap_folded = 1024;
        t->folded = (int64_t *)malloc((size_t)t->cap_folded * sizeof(int64_t));
        t->min_margin = INFINITY;
    }
    return S;
}

void orc_state_free(orc_state *S) {
    if (!S) return;
    int ns = S->cfg.B * S->cfg.Hkv;
    for (int i = 0; i < ns; i++) {
        stream_t *t = &S->st[i];
        free(t->H); free(t->s); pl_free(&t->win); pl_free(&t->sp); free(t->folded);
    }
    free(S->st); free(S->n_tokens); free(S);
}

/* ---- feature map: z_j = sum_i W[i][j] x_i, W is [d][m] row-major, m = D/2 -------------------- */
static void phi_map(const orc_config *c, const float *W, const real *x, real *out) {
    int d = c->d, m = c->D / 2;
    for (int j = 0; j < m; j++) {
        real z = 0;
        for (int i = 0; i < d; i++) z += (real)W[(size_t)i * m + j] * x[i];
        out[j] = z;
    }
    if (c->phi_kind == ORC_PHI_EXP) {
        for (int j = 0; j < m; j++) {
            real z = out[j];
            out[j] = (real)exp((double)z);
            out[m + j] = (real)exp(-(double)z);
        }
    } else {
        /* softmax(z) and softmax(-z), each over the m projections */
        real zmax = out[0], zmin = out[0];
        for (int j = 1; j < m; j++) { if (out[j] > zmax) zmax = out[j]; if (out[j] < zmin) zmin = out[j]; }
        real sp = 0, sn = 0;
        for (int j = 0; j < m; j++) {
            real z = out[j];
            real ep = (real)exp((double)(z - zmax));
            real en = (real)exp((double)(zmin - z));
            out[j] = ep; out[m + j] = en;
            sp += ep; sn += en;
        }
        for (int j = 0; j < m; j++) { out[j] /= sp; out[m + j] /= sn; }
    }
}

/* ---- self-recall error of (k, v) against the current state ---------------------------------- */
static real sre(const orc_config *c, const stream_t *t, const real *phik, const real *v) {
    int d = c->d, D = c->D;
    real den = 0;
    for (int f = 0; f < D; f++) den += phik[f] * t->s[f];
    real acc = 0;
    for (int j = 0; j < d; j++) {
        real pred = 0;
        if (den > 0) {
            real num = 0;
            for (int f = 0; f < D; f++) num += phik[f] * t->H[(size_t)f * d + j];
            pred = num / den;
        }
        real e = pred - v[j];
        acc += e * e;
    }
    return (real)sqrt((double)acc);
}

/* ---- H += phi(k) v^T, s += phi(k) ----------------------------------------------------------- */
static void fold_pair(const orc_config *c, stream_t *t, const real *phik, const real *v, int64_t idx) {
    int d = c->d, D = c->D;
    for (int f = 0; f < D; f++) {
        real p = phik[f];
        real *row = t->H + (size_t)f * d;
        for (int j = 0; j < d; j++) row[j] += p * v[j];
        t->s[f] += p;
    }
    if (t->n_folded == t->cap_folded) {
        t->cap_folded *= 2;
        t->folded = (int64_t *)realloc(t->folded, (size_t)t->cap_folded * sizeof(int64_t));
    }
    t->folded[t->n_folded++] = idx;
}

/*
 * The eligible set E is the sparse cache followed by `n_ev` evicted pairs (already appended to
 * t->sp by the caller, so E == t->sp).  Keep the lambda pairs with the largest SRE under the
 * current state, fold the rest.  `force` (may be NULL) is a list of lambda token indices another
 * implementation kept at this event (-1 = unused slot): if it differs from the oracle's choice
 * only by pairs whose oracle scores lie within tie_eps of each other the oracle adopts it,
 * otherwise the event is counted as a mismatch and the oracle keeps its own choice.
 * Returns the margin SRE_(lambda) - SRE_(lambda+1), or -1 when nothing was scored.
 */
static double select_and_fold(const orc_config *c, stream_t *t, const float *Wk,
                              const int32_t *force, double tie_eps) {
    int d = c->d, D = c->D, lam = c->lambda;
    int n = t->sp.n;
    if (n <= lam) return -1.0;

    real *phis = (real *)malloc((size_t)n * D * sizeof(real));
    real *score = (real *)malloc((size_t)n * sizeof(real));
    int *order = (int *)malloc((size_t)n * sizeof(int));
    char *keep = (char *)calloc((size_t)n, 1);
    for (int e = 0; e < n; e++) {
        phi_map(c, Wk, t->sp.k + (size_t)e * d, phis + (size_t)e * D);
        score[e] = c->score_kind == ORC_SCORE_SRE ? sre(c, t, phis + (size_t)e * D, t->sp.v + (size_t)e * d)
                                                  : t->sp.score[e];
        order[e] = e;
    }
    /* insertion sort by (score descending, token index ascending) */
    for (int a = 1; a < n; a++) {
        int e = order[a], b = a - 1;
        while (b >= 0) {
            int o = order[b];
            int o_first = (score[o] > score[e]) || (score[o] == score[e] && t->sp.idx[o] < t->sp.idx[e]);
            if (o_first) break;
            order[b + 1] = o; b--;
        }
        order[b + 1] = e;
    }
    for (int a = 0; a < lam; a++) keep[order[a]] = 1;
    double margin = lam > 0 ? (double)score[order[lam - 1]] - (double)score[order[lam]] : INFINITY;
    t->n_scored_events++;
    if (margin < t->min_margin) t->min_margin = margin;

    if (force && lam > 0) {
        char *fkeep = (char *)calloc((size_t)n, 1);
        int n_forced = 0, unknown = 0;
        for (int a = 0; a < lam; a++) {
            if (force[a] < 0) continue;
            int found = -1;
            for (int e = 0; e < n; e++) if (t->sp.idx[e] == (int64_t)force[a]) { found = e; break; }
            if (found < 0 || fkeep[found]) unknown = 1; else { fkeep[found] = 1; n_forced++; }
        }
        int differs = 0;
        for (int e = 0; e < n; e++) if (fkeep[e] != keep[e]) differs = 1;
        if (differs) {
            double hi_dropped = -INFINITY, lo_taken = INFINITY; /* own-kept but not forced / forced but not own-kept */
            for (int e = 0; e < n; e++) {
                if (keep[e] && !fkeep[e] && (double)score[e] > hi_dropped) hi_dropped = (double)score[e];
                if (!keep[e] && fkeep[e] && (double)score[e] < lo_taken) lo_taken = (double)score[e];
            }
            /* the band is absolute for the self-recall error (values of order one) and relative for the
               query-dependent scores, whose size depends on eta, the group size and the logits */
            double band = c->score_kind == ORC_SCORE_SRE ? tie_eps : tie_eps * fmax(1.0, fabs(hi_dropped));
            if (!unknown && n_forced == lam && hi_dropped - lo_taken <= band) {
                memcpy(keep, fkeep, (size_t)n);
                t->n_adopted++;
            } else {
                t->n_mismatch++;
            }
        }
        free(fkeep);
    }

    /* fold what is not kept (in eligible-set order), then compact the kept pairs */
    int w = 0;
    for (int e = 0; e < n; e++) {
        if (!keep[e]) {
            fold_pair(c, t, phis + (size_t)e * D, t->sp.v + (size_t)e * d, t->sp.idx[e]);
        }
    }
    for (int e = 0; e < n; e++) {
        if (keep[e]) {
            if (w != e) {
                memcpy(t->sp.k + (size_t)w * d, t->sp.k + (size_t)e * d, d * sizeof(real));
                memcpy(t->sp.v + (size_t)w * d, t->sp.v + (size_t)e * d, d * sizeof(real));
                t->sp.idx[w] = t->sp.idx[e];
                t->sp.score[w] = t->sp.score[e];
            }
            w++;
        }
    }
    t->sp.n = w;
    free(phis); free(score); free(order); free(keep);
    return margin;
}

/* One query's contribution to the score of one key (appendix "scoring ablation"). */
static real query_term(const orc_config *c, const real *phiq, const real *q, const real *phik, const real *k) {
    real dot = 0, a = 0;
    for (int j = 0; j < c->d; j++) dot += q[j] * k[j];
    for (int f = 0; f < c->D; f++) a += phiq[f] * phik[f];
    real w = (real)exp((double)((real)c->scale * dot));
    switch (c->score_kind) {
        case ORC_SCORE_WERR_SQ: return (w - a) * (w - a);
        case ORC_SCORE_WERR_ABS: return (real)fabs((double)(w - a));
        case ORC_SCORE_OVEREST: return a / w;
        default: return w; /* ORC_SCORE_ATTN */
    }
}

/*
 * Query q with token index tq adds its term to every pair it sees inside the sliding-window band
 * tq-eta+1 .. tq: pairs of the window list and the first n_extra rows of the current chunk (token
 * indices tok0 .. ; their sums are kept in xscore until the chunk joins the window).
 */
static void accumulate_scores(const orc_config *c, stream_t *t, const float *Wq, const float *Wk, const real *q,
                              int64_t tq, const real *xk, int n_extra, int64_t tok0, real *xscore) {
    if (c->score_kind == ORC_SCORE_SRE) return;
    int d = c->d, D = c->D;
    real *phiq = (real *)malloc((size_t)D * sizeof(real));
    real *phik = (real *)malloc((size_t)D * sizeof(real));
    phi_map(c, Wq, q, phiq);
    for (int i = 0; i < t->win.n; i++) {
        if (t->win.idx[i] < tq - c->eta + 1 || t->win.idx[i] > tq) continue;
        phi_map(c, Wk, t->win.k + (size_t)i * d, phik);
        t->win.score[i] += query_term(c, phiq, q, phik, t->win.k + (size_t)i * d);
    }
    for (int i = 0; i < n_extra; i++) {
        if (tok0 + i < tq - c->eta + 1 || tok0 + i > tq) continue;
        phi_map(c, Wk, xk + (size_t)i * d, phik);
        xscore[i] += query_term(c, phiq, q, phik, xk + (size_t)i * d);
    }
    free(phiq); free(phik);
}

/*
 * y = [phi(q)^T H + sum_i exp(scale q.k_i) v_i] / [phi(q)^T s + sum_i exp(scale q.k_i)]
 * over the sparse cache, the window, and the first n_extra rows of (xk, xv) (the causal part of
 * the current chunk during prefill; n_extra = 0 in decode).  With cfg.hide the hidden-state terms
 * and / or the sparse-cache terms are left out of both sums.
 */
static void attend(const orc_config *c, const stream_t *t, const float *Wq, const real *q,
                   const real *xk, const real *xv, int n_extra, double *out) {
    int d = c->d, D = c->D;
    real *phiq = (real *)malloc((size_t)D * sizeof(real));
    real *num = (real *)calloc((size_t)d, sizeof(real));
    real den = 0;
    phi_map(c, Wq, q, phiq);
    if (!(c->hide & 1)) {
        for (int f = 0; f < D; f++) {
            real p = phiq[f];
            const real *row = t->H + (size_t)f * d;
            for (int j = 0; j < d; j++) num[j] += p * row[j];
            den += p * t->s[f];
        }
    }
    const pair_list *lists[2] = { &t->sp, &t->win };
    for (int l = (c->hide & 2) ? 1 : 0; l < 2; l++) {
        const pair_list *p = lists[l];
        for (int i = 0; i < p->n; i++) {
            real dot = 0;
            for (int j = 0; j < d; j++) dot += q[j] * p->k[(size_t)i * d + j];
            real w = (real)exp((double)((real)c->scale * dot));
            for (int j = 0; j < d; j++) num[j] += w * p->v[(size_t)i * d + j];
            den += w;
        }
    }
    for (int i = 0; i < n_extra; i++) {
        real dot = 0;
        for (int j = 0; j < d; j++) dot += q[j] * xk[(size_t)i * d + j];
        real w = (real)exp((double)((real)c->scale * dot));
        for (int j = 0; j < d; j++) num[j] += w * xv[(size_t)i * d + j];
        den += w;
    }
    for (int j = 0; j < d; j++) out[j] = (double)(num[j] / den);
    free(phiq); free(num);
}

static void load_row(real *dst, const float *src, int d) { for (int j = 0; j < d; j++) dst[j] = (real)src[j]; }

/*
 * One generation step for every sequence of the batch.
 * q [B,Hq,d], k, v [B,Hkv,d] (float holding storage-type values), Wq [Hq,d,m], Wk [Hkv,d,m],
 * out [B,Hq,d] double.  force_sel [B,Hkv,lambda] or NULL.  margin_out [B,Hkv] or NULL.
 */
int orc_decode_step(orc_state *S, const float *q, const float *k, const float *v,
                    const float *Wq, const float *Wk, double *out,
                    const int32_t *force_sel, double tie_eps, double *margin_out) {
    if (!S || !q || !k || !v || !Wq || !Wk || !out) return -1;
    const orc_config *c = &S->cfg;
    int d = c->d, m = c->D / 2, g = c->Hq / c->Hkv, ns = c->B * c->Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int si = 0; si < ns; si++) {
        int b = si / c->Hkv, h = si % c->Hkv;
        stream_t *t = &S->st[si];
        const float *Wk_h = Wk + (size_t)h * d * m;
        int64_t tok = S->n_tokens[b];
        real *kr = (real *)malloc((size_t)d * sizeof(real));
        real *vr = (real *)malloc((size_t)d * sizeof(real));
        load_row(kr, k + (size_t)si * d, d);
        load_row(vr, v + (size_t)si * d, d);
        /* 1. the new pair enters the window; the oldest leaves once it holds more than eta */
        pl_push(&t->win, d, kr, vr, tok);
        double margin = -1.0;
        if (t->win.n > c->eta) {
            /* 2. E = G u {leaving pair}; keep top-lambda, fold the rest */
            pl_push_scored(&t->sp, d, t->win.k, t->win.v, t->win.idx[0], t->win.score[0]);
            pl_drop_front(&t->win, d, 1);
            margin = select_and_fold(c, t, Wk_h, force_sel ? force_sel + (size_t)si * c->lambda : NULL, tie_eps);
        }
        if (margin_out) margin_out[si] = margin;
        /* 3. outputs of the group's query heads with the updated memories */
        for (int r = 0; r < g; r++) {
            int hq = h * g + r;
            load_row(kr, q + ((size_t)b * c->Hq + hq) * d, d);
            attend(c, t, Wq + (size_t)hq * d * m, kr, NULL, NULL, 0, out + ((size_t)b * c->Hq + hq) * d);
            accumulate_scores(c, t, Wq + (size_t)hq * d * m, Wk_h, kr, tok, NULL, 0, 0, NULL);
        }
        free(kr); free(vr);
    }
    for (int b = 0; b < c->B; b++) S->n_tokens[b] += 1;
    return 0;
}

/*
 * Chunkwise prefill of T tokens for every sequence.
 * q [B,Hq,T,d] (may be NULL together with out: caches are updated, no outputs are produced),
 * k, v [B,Hkv,T,d], out [B,Hq,T,d] double.
 * force_sel / sel_log [B,Hkv,n_chunks,lambda] (NULL allowed), margin_log [B,Hkv,n_chunks] (NULL
 * allowed), n_chunks = ceil(T / C).  sel_log receives the token indices kept after each chunk
 * (ascending, -1 padded).
 */
int orc_prefill(orc_state *S, const float *q, const float *k, const float *v,
                const float *Wq, const float *Wk, int T, double *out,
                const int32_t *force_sel, double tie_eps, int32_t *sel_log, double *margin_log) {
    if (!S || !k || !v || !Wk || T < 0) return -1;
    if ((q == NULL) != (out == NULL)) return -1;
    if (!q && S->cfg.score_kind != ORC_SCORE_SRE && T > 0) return -1; /* these scores are sums over queries */
    if (q && !Wq) return -1;
    const orc_config *c = &S->cfg;
    int d = c->d, m = c->D / 2, g = c->Hq / c->Hkv, ns = c->B * c->Hkv, C = c->C, lam = c->lambda;
    int n_chunks = (T + C - 1) / C;
#pragma omp parallel for schedule(dynamic, 1)
    for (int si = 0; si < ns; si++) {
        int b = si / c->Hkv, h = si % c->Hkv;
        stream_t *t = &S->st[si];
        const float *Wk_h = Wk + (size_t)h * d * m;
        real *ck = (real *)malloc((size_t)C * d * sizeof(real));
        real *cv = (real *)malloc((size_t)C * d * sizeof(real));
        real *qr = (real *)malloc((size_t)d * sizeof(real));
        real *cs = (real *)malloc((size_t)C * sizeof(real));
        for (int j = 0; j < n_chunks; j++) {
            int a = j * C, cl = (T - a < C) ? T - a : C;
            int64_t tok0 = S->n_tokens[b] + a;
            for (int i = 0; i < cl; i++) {
                load_row(ck + (size_t)i * d, k + ((size_t)si * T + a + i) * d, d);
                load_row(cv + (size_t)i * d, v + ((size_t)si * T + a + i) * d, d);
                cs[i] = 0;
            }
            /* 1. outputs: entry state, entry sparse cache, entry window, own chunk causally */
            if (q) {
                for (int r = 0; r < g; r++) {
                    int hq = h * g + r;
                    for (int i = 0; i < cl; i++) {
                        size_t off = (((size_t)b * c->Hq + hq) * T + a + i) * d;
                        load_row(qr, q + off, d);
                        attend(c, t, Wq + (size_t)hq * d * m, qr, ck, cv, i + 1, out + off);
                        accumulate_scores(c, t, Wq + (size_t)hq * d * m, Wk_h, qr, tok0 + i, ck, i + 1, tok0, cs);
                    }
                }
            }
            /* 2. the chunk joins the window; what no longer fits is the evicted group */
            for (int i = 0; i < cl; i++) pl_push_scored(&t->win, d, ck + (size_t)i * d, cv + (size_t)i * d, tok0 + i, cs[i]);
            int n_ev = t->win.n - c->eta;
            double margin = -1.0;
            if (n_ev > 0) {
                for (int i = 0; i < n_ev; i++)
                    pl_push_scored(&t->sp, d, t->win.k + (size_t)i * d, t->win.v + (size_t)i * d, t->win.idx[i], t->win.score[i]);
                pl_drop_front(&t->win, d, n_ev);
                const int32_t *f = force_sel ? force_sel + ((size_t)si * n_chunks + j) * lam : NULL;
                margin = select_and_fold(c, t, Wk_h, f, tie_eps);
            }
            if (margin_log) margin_log[(size_t)si * n_chunks + j] = margin;
            if (sel_log) {
                int32_t *dst = sel_log + ((size_t)si * n_chunks + j) * lam;
                for (int a2 = 0; a2 < lam; a2++) dst[a2] = -1;
                for (int a2 = 0; a2 < t->sp.n; a2++) dst[a2] = (int32_t)t->sp.idx[a2];
                /* ascending order */
                for (int x = 1; x < t->sp.n; x++) {
                    int32_t e = dst[x]; int y = x - 1;
                    while (y >= 0 && dst[y] > e) { dst[y + 1] = dst[y]; y--; }
                    dst[y + 1] = e;
                }
            }
        }
        free(ck); free(cv); free(qr); free(cs);
    }
    for (int b = 0; b < c->B; b++) S->n_tokens[b] += T;
    return 0;
}

/* ---- accessors (tests read the state through these) ----------------------------------------- */

void orc_get_H(const orc_state *S, double *out) { /* [B,Hkv,D,d] */
    const orc_config *c = &S->cfg; size_t n = (size_t)c->D * c->d;
    for (int si = 0; si < c->B * c->Hkv; si++)
        for (size_t i = 0; i < n; i++) out[(size_t)si * n + i] = (double)S->st[si].H[i];
}
void orc_get_s(const orc_state *S, double *out) { /* [B,Hkv,D] */
    const orc_config *c = &S->cfg;
    for (int si = 0; si < c->B * c->Hkv; si++)
        for (int i = 0; i < c->D; i++) out[(size_t)si * c->D + i] = (double)S->st[si].s[i];
}
static void sorted_idx(const pair_list *p, int32_t *dst, int cap) {
    for (int a = 0; a < cap; a++) dst[a] = -1;
    for (int a = 0; a < p->n && a < cap; a++) dst[a] = (int32_t)p->idx[a];
    for (int x = 1; x < p->n && x < cap; x++) {
        int32_t e = dst[x]; int y = x - 1;
        while (y >= 0 && dst[y] > e) { dst[y + 1] = dst[y]; y--; }
        dst[y + 1] = e;
    }
}
void orc_get_sparse_idx(const orc_state *S, int32_t *out) { /* [B,Hkv,lambda] ascending, -1 padded */
    const orc_config *c = &S->cfg;
    for (int si = 0; si < c->B * c->Hkv; si++) sorted_idx(&S->st[si].sp, out + (size_t)si * c->lambda, c->lambda);
}
void orc_get_window_idx(const orc_state *S, int32_t *out) { /* [B,Hkv,eta] ascending, -1 padded */
    const orc_config *c = &S->cfg;
    for (int si = 0; si < c->B * c->Hkv; si++) sorted_idx(&S->st[si].win, out + (size_t)si * c->eta, c->eta);
}
/* sparse / window pairs of one stream in storage order: k,v [n][d] double, idx [n]; returns n */
int orc_get_pairs(const orc_state *S, int stream, int which /*0 sparse, 1 window*/, double *k, double *v, int64_t *idx) {
    const orc_config *c = &S->cfg;
    const pair_list *p = which ? &S->st[stream].win : &S->st[stream].sp;
    for (int i = 0; i < p->n; i++) {
        for (int j = 0; j < c->d; j++) {
            if (k) k[(size_t)i * c->d + j] = (double)p->k[(size_t)i * c->d + j];
            if (v) v[(size_t)i * c->d + j] = (double)p->v[(size_t)i * c->d + j];
        }
        if (idx) idx[i] = p->idx[i];
    }
    return p->n;
}
/* query-dependent scores gathered so far by the sparse / window pairs of one stream, same order as orc_get_pairs */
int orc_get_scores(const orc_state *S, int stream, int which, double *out) {
    const pair_list *p = which ? &S->st[stream].win : &S->st[stream].sp;
    for (int i = 0; i < p->n; i++) out[i] = (double)p->score[i];
    return p->n;
}
int64_t orc_get_folded(const orc_state *S, int stream, int64_t *out, int64_t cap) {
    const stream_t *t = &S->st[stream];
    for (int64_t i = 0; i < t->n_folded && i < cap; i++) out[i] = t->folded[i];
    return t->n_folded;
}
int64_t orc_get_n_tokens(const orc_state *S, int b) { return S->n_tokens[b]; }
/* totals over all streams: [scored events, adopted, mismatches]; returns the smallest margin seen */
double orc_get_stats(const orc_state *S, int64_t *out3) {
    const orc_config *c = &S->cfg; double mm = INFINITY;
    out3[0] = out3[1] = out3[2] = 0;
    for (int si = 0; si < c->B * c->Hkv; si++) {
        out3[0] += S->st[si].n_scored_events; out3[1] += S->st[si].n_adopted; out3[2] += S->st[si].n_mismatch;
        if (S->st[si].min_margin < mm) mm = S->st[si].min_margin;
    }
    return mm;
}

/*
 * Overwrite one stream's memories (used to restart the oracle from a state produced elsewhere).
 * H [D,d], s [D] double; sparse and window pairs as float rows with their token indices, the
 * window in chronological order.  The folded list is cleared (its content is unknown).
 */
int orc_set_stream(orc_state *S, int stream, const double *H, const double *s,
                   const float *spk, const float *spv, const int64_t *spidx, int spn,
                   const float *wk, const float *wv, const int64_t *widx, int wn) {
    const orc_config *c = &S->cfg;
    if (stream < 0 || stream >= c->B * c->Hkv || spn > c->lambda || wn > c->eta) return -1;
    stream_t *t = &S->st[stream];
    for (size_t i = 0; i < (size_t)c->D * c->d; i++) t->H[i] = (real)H[i];
    for (int i = 0; i < c->D; i++) t->s[i] = (real)s[i];
    real *kr = (real *)malloc((size_t)c->d * sizeof(real)), *vr = (real *)malloc((size_t)c->d * sizeof(real));
    t->sp.n = 0; t->win.n = 0; t->n_folded = 0;
    for (int i = 0; i < spn; i++) {
        load_row(kr, spk + (size_t)i * c->d, c->d); load_row(vr, spv + (size_t)i * c->d, c->d);
        pl_push(&t->sp, c->d, kr, vr, spidx[i]);
    }
    for (int i = 0; i < wn; i++) {
        load_row(kr, wk + (size_t)i * c->d, c->d); load_row(vr, wv + (size_t)i * c->d, c->d);
        pl_push(&t->win, c->d, kr, vr, widx[i]);
    }
    free(kr); free(vr);
    return 0;
}
void orc_set_n_tokens(orc_state *S, int b, int64_t n) { S->n_tokens[b] = n; }

/* ---- probes used by the pins ----------------------------------------------------------------- */

/* phi(x) for one vector under configuration (d, D, phi_kind); W [d][D/2], x [d], out [D] */
void orc_phi(const orc_config *cfg, const float *W, const double *x, double *out) {
    real *xr = (real *)malloc((size_t)cfg->d * sizeof(real));
    real *o = (real *)malloc((size_t)cfg->D * sizeof(real));
    for (int i = 0; i < cfg->d; i++) xr[i] = (real)x[i];
    phi_map(cfg, W, xr, o);
    for (int i = 0; i < cfg->D; i++) out[i] = (double)o[i];
    free(xr); free(o);
}
/* SRE of an arbitrary pair against the present state of one stream */
double orc_sre_probe(const orc_state *S, int stream, const float *Wk_h, const double *k, const double *v) {
    const orc_config *c = &S->cfg;
    real *kr = (real *)malloc((size_t)c->d * sizeof(real)), *vr = (real *)malloc((size_t)c->d * sizeof(real));
    real *p = (real *)malloc((size_t)c->D * sizeof(real));
    for (int i = 0; i < c->d; i++) { kr[i] = (real)k[i]; vr[i] = (real)v[i]; }
    phi_map(c, Wk_h, kr, p);
    double r = (double)sre(c, &S->st[stream], p, vr);
    free(kr); free(vr); free(p);
    return r;
}

/*
 * Elements stored per head after t tokens: the smaller of a plain KV cache, t (d_k + d_v), and
 * the three memory systems, (w + lambda)(d_k + d_v) + D d_v + D, where the local cache holds
 * w = 2 eta pairs during chunkwise inference (two chunks) and eta pairs in generation.
 */
int64_t orc_cache_elems(int64_t t, int64_t eta, int64_t lambda, int64_t dk, int64_t dv, int64_t D, int two_chunks) {
    int64_t plain = t * (dk + dv);
    int64_t w = two_chunks ? 2 * eta : eta;
    int64_t lola = (w + lambda) * (dk + dv) + D * dv + D;
    return plain < lola ? plain : lola;
}

int orc_real_bytes(void) { return (int)sizeof(real); }

/* threads the parallel loops over streams will use (for reporting the CPU baseline) */
int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
