/*
 * wgkv_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, single-purpose CPU reference for the Write-Gated KV hot path
 * ("KV Admission: Learning What to Write for Efficient Long-Context LLM
 * Inference").  It exists so that the GPU library can be checked against
 * something written straight from the paper.  It shares no code, header, table
 * or helper with the GPU library, and only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.
 *
 * Two halves that must agree with each other:
 *
 *  (1) the DEFINITION of the result: attention of a query at position i over
 *      the keys j <= i that the vertical-slash mask leaves visible,
 *        M_ij = (1(i-j < W_local) or 1(g_j >= tau)) and 1(i >= j)
 *      (Sec. 4.2 "Vertical-slash sparse attention", mask equation) applied to
 *      scaled-dot-product attention (Sec. 2.1 equation; Sec. 3.2 first
 *      equation of "Write-Gated Attention").  This half keeps the whole,
 *      undropped K/V/g history and never looks at rings, pages or pointers.
 *
 *  (2) the MECHANISM that the system section describes, simulated one token
 *      at a time with ordinary arrays: a ring-buffer local cache of W_local
 *      slots, a growing global cache, per-head page tables onto one physical
 *      pool (Sec. 4.1), initial cache population (Sec. 4.2) and lazy promotion
 *      (Sec. 4.3, steps (1)-(3)).
 *
 *  (3) budgeted eviction on the global cache (the appendix on the synergy with
 *      eviction): importance scores from an observation window and removal of
 *      the lowest-scored entries with compaction and release of pages.
 *
 *  (4) read-time page selection with key landmarks over the admitted cache (the
 *      appendix on the synergy with selection) and attention over the selection.
 *
 *  (5) the gates that produce the scores: the linear gate of the chunked-prefill
 *      workload and the Write-Gate MLP of Sec. 3.2.
 *
 *  (6) the training-time attention with the soft gate as a log-space bias
 *      (Sec. 3.2, "Write-Gated Attention" and "Log-space transformation"), forward
 *      and the gradients with respect to q, k, v and the gate scores (at the end of
 *      the file).
 *
 * All floating-point work is done in double; inputs arrive as float (the
 * exact widening of bf16 or fp32 data).  Threshold tests are done on the
 * stored fp32 score with the C `>=` operator, so a NaN score never admits.
 *
 * Readings where the paper is silent (the same list is in the design notes):
 *  - ring slot of position p is p mod W_local; the local pointer is t mod W.
 *  - the window contains the token itself (i-j < W with j <= i).
 *  - the global cache is ordered by position (victims leave in order).
 *  - the ring stores the fp32 score; the tau of the evicting call decides.
 *  - attention in decode is taken after the write of the new token.
 *  - pages: a LIFO free stack, free_stack[i] = n_pages-1-i, pop takes
 *    free_stack[--free_top].  Within one call page demands are served unit by
 *    unit, units ordered by (position of the sequence in the call, kv head);
 *    a unit's ceil(W/P) local pages are taken at its first use, before any of
 *    its global pages.  This rule is this project's own: the paper fixes no
 *    allocation order, so physical page ids are "parity unpinned" with
 *    respect to the paper; everything else below is pinned by the tests.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_ERR_ARG (-1)
#define ORC_ERR_OUT_OF_PAGES (-2)
#define ORC_ERR_PT_OVERFLOW (-3)
#define ORC_ERR_NOMEM (-4)

typedef struct {
    int32_t n_layers, n_q_heads, n_kv_heads, head_dim;
    int32_t page_size, w_local, max_seqs, max_global_pages;
    int64_t n_pages;
    int32_t keep_payload; /* 0: integer state only (scores, positions, pages) */
} orc_config;

typedef struct {
    int64_t glen, gcap;
    int64_t *gpos;        /* position of every global entry, ascending */
    float *gk, *gv;       /* [gcap][d] when payload is kept            */
    float *ring_g;        /* [W] stored score of the slot's token      */
    int64_t *ring_pos;    /* [W] position held by the slot, -1 = empty */
    float *ring_k, *ring_v; /* [W][d] when payload is kept            */
    int32_t *local_pt;    /* [ceil(W/P)]                               */
    int32_t *global_pt;   /* [max_global_pages], -1 = unused           */
} orc_head;

typedef struct {
    int64_t t;     /* tokens seen so far by this (sequence, layer) */
    int touched;   /* local pages handed out                        */
    orc_head *h;   /* [n_kv_heads]                                  */
} orc_sl;

typedef struct {
    orc_config c;
    int n_local_pages;
    orc_sl *sl; /* [max_seqs][n_layers] */
    int32_t *free_stack;
    int64_t free_top;
} orc_state;

static orc_sl *get_sl(orc_state *S, int seq, int layer) {
    return &S->sl[(size_t)seq * S->c.n_layers + layer];
}

int orc_n_local_pages(const orc_state *S) { return S->n_local_pages; }

void orc_destroy(orc_state *S) {
    if (!S) return;
    if (S->sl) {
        size_t n = (size_t)S->c.max_seqs * S->c.n_layers;
        for (size_t i = 0; i < n; i++) {
            if (!S->sl[i].h) continue;
            for (int h = 0; h < S->c.n_kv_heads; h++) {
                orc_head *H = &S->sl[i].h[h];
                free(H->gpos); free(H->gk); free(H->gv);
                free(H->ring_g); free(H->ring_pos);
                free(H->ring_k); free(H->ring_v);
                free(H->local_pt); free(H->global_pt);
            }
            free(S->sl[i].h);
        }
        free(S->sl);
    }
    free(S->free_stack);
    free(S);
}

static void reset_head(orc_state *S, orc_head *H) {
    const int W = S->c.w_local;
    H->glen = 0;
    for (int s = 0; s < W; s++) { H->ring_g[s] = 0.0f; H->ring_pos[s] = -1; }
    for (int i = 0; i < S->n_local_pages; i++) H->local_pt[i] = -1;
    for (int i = 0; i < S->c.max_global_pages; i++) H->global_pt[i] = -1;
}

orc_state *orc_create(const orc_config *c) {
    if (!c || c->n_layers < 1 || c->n_kv_heads < 1 || c->n_q_heads < c->n_kv_heads ||
        c->n_q_heads % c->n_kv_heads || c->head_dim < 1 || c->page_size < 1 ||
        c->w_local < 1 || c->max_seqs < 1 || c->max_global_pages < 0 || c->n_pages < 0)
        return NULL;
    orc_state *S = (orc_state *)calloc(1, sizeof(orc_state));
    if (!S) return NULL;
    S->c = *c;
    S->n_local_pages = (c->w_local + c->page_size - 1) / c->page_size;
    size_t n = (size_t)c->max_seqs * c->n_layers;
    S->sl = (orc_sl *)calloc(n, sizeof(orc_sl));
    S->free_stack = (int32_t *)malloc(sizeof(int32_t) * (size_t)(c->n_pages > 0 ? c->n_pages : 1));
    if (!S->sl || !S->free_stack) { orc_destroy(S); return NULL; }
    for (int64_t i = 0; i < c->n_pages; i++) S->free_stack[i] = (int32_t)(c->n_pages - 1 - i);
    S->free_top = c->n_pages;
    const int W = c->w_local, d = c->head_dim;
    for (size_t i = 0; i < n; i++) {
        S->sl[i].h = (orc_head *)calloc((size_t)c->n_kv_heads, sizeof(orc_head));
        if (!S->sl[i].h) { orc_destroy(S); return NULL; }
        for (int h = 0; h < c->n_kv_heads; h++) {
            orc_head *H = &S->sl[i].h[h];
            H->ring_g = (float *)malloc(sizeof(float) * W);
            H->ring_pos = (int64_t *)malloc(sizeof(int64_t) * W);
            H->local_pt = (int32_t *)malloc(sizeof(int32_t) * S->n_local_pages);
            H->global_pt = (int32_t *)malloc(sizeof(int32_t) * (size_t)(c->max_global_pages > 0 ? c->max_global_pages : 1));
            if (c->keep_payload) {
                H->ring_k = (float *)calloc((size_t)W * d, sizeof(float));
                H->ring_v = (float *)calloc((size_t)W * d, sizeof(float));
            }
            if (!H->ring_g || !H->ring_pos || !H->local_pt || !H->global_pt ||
                (c->keep_payload && (!H->ring_k || !H->ring_v))) { orc_destroy(S); return NULL; }
            reset_head(S, H);
        }
    }
    return S;
}

static int pop_page(orc_state *S, int32_t *page) {
    if (S->free_top <= 0) return ORC_ERR_OUT_OF_PAGES;
    *page = S->free_stack[--S->free_top];
    return ORC_OK;
}

/* Sec. 4.3 steps (1)-(3) for one head: look at the victim under the local
 * pointer, promote it when its stored score passes the threshold, then let the
 * new token take the slot.  Position p is the new token's; the victim, if the
 * ring is already full, is position p - W. */
static int push_one(orc_state *S, orc_head *H, int64_t p, const float *k, const float *v,
                    float g, float tau, int *promoted) {
    const int W = S->c.w_local, P = S->c.page_size, d = S->c.head_dim;
    const int s = (int)(p % W); /* local pointer */
    *promoted = 0;
    if (p >= W) {
        if (H->ring_g[s] >= tau) { /* victim passes the gate */
            if (H->glen % P == 0) { /* the global pointer enters a new page */
                int64_t lp = H->glen / P;
                if (lp >= S->c.max_global_pages) return ORC_ERR_PT_OVERFLOW;
                int32_t page;
                int rc = pop_page(S, &page);
                if (rc) return rc;
                H->global_pt[lp] = page;
            }
            if (H->glen == H->gcap) {
                int64_t nc = H->gcap ? H->gcap * 2 : 64;
                int64_t *np_ = (int64_t *)realloc(H->gpos, sizeof(int64_t) * nc);
                if (!np_) return ORC_ERR_NOMEM;
                H->gpos = np_;
                if (S->c.keep_payload) {
                    float *nk = (float *)realloc(H->gk, sizeof(float) * nc * d);
                    if (!nk) return ORC_ERR_NOMEM;
                    H->gk = nk;
                    float *nv = (float *)realloc(H->gv, sizeof(float) * nc * d);
                    if (!nv) return ORC_ERR_NOMEM;
                    H->gv = nv;
                }
                H->gcap = nc;
            }
            H->gpos[H->glen] = H->ring_pos[s];
            if (S->c.keep_payload) {
                memcpy(H->gk + H->glen * d, H->ring_k + (size_t)s * d, sizeof(float) * d);
                memcpy(H->gv + H->glen * d, H->ring_v + (size_t)s * d, sizeof(float) * d);
            }
            H->glen += 1; /* global pointer advances */
            *promoted = 1;
        }
        /* else: the victim leaves the window unadmitted and is gone */
    }
    H->ring_g[s] = g;
    H->ring_pos[s] = p;
    if (S->c.keep_payload) {
        memcpy(H->ring_k + (size_t)s * d, k, sizeof(float) * d);
        memcpy(H->ring_v + (size_t)s * d, v, sizeof(float) * d);
    }
    return ORC_OK;
}

/*
 * Feed tokens to one layer of several sequences.  Prefill (Sec. 4.2 "Initial
 * cache population"), a prefill chunk and a decode step (Sec. 4.3) are all the
 * same thing here: n_tokens[b] pushes for sequence seq_ids[b].
 *   k, v : [sum n_tokens][n_kv_heads][d] floats (NULL allowed without payload)
 *   g    : [sum n_tokens][n_kv_heads] scores
 *   admit_out    (optional) [sum n_tokens][n_kv_heads]: 1(g >= tau)  (Sec. 3.3, last sentence)
 *   promoted_out (optional) same shape: 1 when the push of that token moved
 *                its victim into the global cache.
 */
int orc_push_tokens(orc_state *S, int layer, int n_seqs, const int32_t *seq_ids,
                    const int32_t *n_tokens, const float *k, const float *v, const float *g,
                    float tau, uint8_t *admit_out, uint8_t *promoted_out) {
    if (!S || layer < 0 || layer >= S->c.n_layers || n_seqs < 0) return ORC_ERR_ARG;
    const int Hk = S->c.n_kv_heads, d = S->c.head_dim;
    if (S->c.keep_payload && (!k || !v)) return ORC_ERR_ARG;
    int64_t base = 0;
    for (int b = 0; b < n_seqs; b++) {
        int seq = seq_ids[b];
        if (seq < 0 || seq >= S->c.max_seqs || n_tokens[b] < 0) return ORC_ERR_ARG;
        for (int b2 = 0; b2 < b; b2++) if (seq_ids[b2] == seq) return ORC_ERR_ARG;
        base += n_tokens[b];
    }
    base = 0;
    for (int b = 0; b < n_seqs; b++) {
        orc_sl *sl = get_sl(S, seq_ids[b], layer);
        const int T = n_tokens[b];
        for (int h = 0; h < Hk; h++) {
            orc_head *H = &sl->h[h];
            if (!sl->touched && T > 0) {
                for (int i = 0; i < S->n_local_pages; i++) {
                    int rc = pop_page(S, &H->local_pt[i]);
                    if (rc) return rc;
                }
            }
            for (int i = 0; i < T; i++) {
                size_t row = (size_t)(base + i) * Hk + h;
                int promoted = 0;
                int rc = push_one(S, H, sl->t + i, k ? k + row * d : NULL, v ? v + row * d : NULL,
                                  g[row], tau, &promoted);
                if (rc) return rc;
                if (admit_out) admit_out[row] = (uint8_t)(g[row] >= tau);
                if (promoted_out) promoted_out[row] = (uint8_t)promoted;
            }
        }
        if (T > 0) sl->touched = 1;
        sl->t += T;
        base += T;
    }
    return ORC_OK;
}

/* Give every page of a sequence slot back: layers ascending, kv heads
 * ascending, a unit's local pages then its global pages, each ascending. */
int orc_free_seq(orc_state *S, int seq) {
    if (!S || seq < 0 || seq >= S->c.max_seqs) return ORC_ERR_ARG;
    const int P = S->c.page_size;
    for (int l = 0; l < S->c.n_layers; l++) {
        orc_sl *sl = get_sl(S, seq, l);
        for (int h = 0; h < S->c.n_kv_heads; h++) {
            orc_head *H = &sl->h[h];
            if (sl->touched) {
                for (int i = 0; i < S->n_local_pages; i++) S->free_stack[S->free_top++] = H->local_pt[i];
                int64_t ngp = (H->glen + P - 1) / P;
                for (int64_t i = 0; i < ngp; i++) S->free_stack[S->free_top++] = H->global_pt[i];
            }
            reset_head(S, H);
        }
        sl->t = 0;
        sl->touched = 0;
    }
    return ORC_OK;
}

/* ---- state read-out (for bit-exact comparison) ---- */

int64_t orc_seq_len(const orc_state *S, int seq, int layer) {
    return S->sl[(size_t)seq * S->c.n_layers + layer].t;
}
int64_t orc_global_len(const orc_state *S, int seq, int layer, int h) {
    return S->sl[(size_t)seq * S->c.n_layers + layer].h[h].glen;
}
int64_t orc_free_top(const orc_state *S) { return S->free_top; }
void orc_get_free_stack(const orc_state *S, int32_t *out) {
    memcpy(out, S->free_stack, sizeof(int32_t) * (size_t)S->c.n_pages);
}
void orc_get_head_tables(const orc_state *S, int seq, int layer, int h, int32_t *local_pt,
                         int32_t *global_pt, float *ring_g, int64_t *ring_pos) {
    const orc_head *H = &S->sl[(size_t)seq * S->c.n_layers + layer].h[h];
    if (local_pt) memcpy(local_pt, H->local_pt, sizeof(int32_t) * S->n_local_pages);
    if (global_pt) memcpy(global_pt, H->global_pt, sizeof(int32_t) * (size_t)S->c.max_global_pages);
    if (ring_g) memcpy(ring_g, H->ring_g, sizeof(float) * S->c.w_local);
    if (ring_pos) memcpy(ring_pos, H->ring_pos, sizeof(int64_t) * S->c.w_local);
}
void orc_get_global_pos(const orc_state *S, int seq, int layer, int h, int64_t *out) {
    const orc_head *H = &S->sl[(size_t)seq * S->c.n_layers + layer].h[h];
    if (H->glen > 0) memcpy(out, H->gpos, sizeof(int64_t) * (size_t)H->glen);  /* empty cache: no array yet */
}
/* cached rows: global entries in order, then ring slots 0..W-1 */
int orc_get_payload(const orc_state *S, int seq, int layer, int h, float *gk, float *gv,
                    float *ring_k, float *ring_v) {
    if (!S->c.keep_payload) return ORC_ERR_ARG;
    const orc_head *H = &S->sl[(size_t)seq * S->c.n_layers + layer].h[h];
    const size_t d = S->c.head_dim;
    if (gk && H->glen > 0) memcpy(gk, H->gk, sizeof(float) * H->glen * d);
    if (gv && H->glen > 0) memcpy(gv, H->gv, sizeof(float) * H->glen * d);
    if (ring_k) memcpy(ring_k, H->ring_k, sizeof(float) * S->c.w_local * d);
    if (ring_v) memcpy(ring_v, H->ring_v, sizeof(float) * S->c.w_local * d);
    return ORC_OK;
}

/* ---- attention ---- */

/* softmax(scores) . V for one query head, everything in double, max-subtracted
 * (Sec. 2.1 equation).  rows[n] point at the K and V vectors of the keys.  */
static void softmax_av(const float *q, const float *const *krows, const float *const *vrows,
                       int64_t n, int d, double scale, double *scores, double *out) {
    double mx = -INFINITY;
    for (int64_t j = 0; j < n; j++) {
        double s = 0.0;
        for (int e = 0; e < d; e++) s += (double)q[e] * (double)krows[j][e];
        s *= scale;
        scores[j] = s;
        if (s > mx) mx = s;
    }
    double den = 0.0;
    for (int64_t j = 0; j < n; j++) { scores[j] = exp(scores[j] - mx); den += scores[j]; }
    for (int e = 0; e < d; e++) out[e] = 0.0;
    for (int64_t j = 0; j < n; j++) {
        double w = scores[j] / den;
        for (int e = 0; e < d; e++) out[e] += w * (double)vrows[j][e];
    }
}

/* Mechanism attention for one sequence/layer after the pushes so far: every
 * query head of a group reads its kv head's global entries and valid ring
 * slots (Sec. 4.3, last sentence).  q: [n_q_heads][d], out: [n_q_heads][d]. */
int orc_attend_cached(const orc_state *S, int seq, int layer, const float *q, double scale,
                      double *out) {
    if (!S || !S->c.keep_payload) return ORC_ERR_ARG;
    const int Hq = S->c.n_q_heads, Hk = S->c.n_kv_heads, d = S->c.head_dim, W = S->c.w_local;
    const int G = Hq / Hk;
    const orc_sl *sl = &S->sl[(size_t)seq * S->c.n_layers + layer];
    for (int h = 0; h < Hk; h++) {
        const orc_head *H = &sl->h[h];
        int64_t n = H->glen;
        for (int s = 0; s < W; s++) if (H->ring_pos[s] >= 0) n++;
        if (n == 0) { /* nothing cached: define the output as zero */
            for (int qh = h * G; qh < (h + 1) * G; qh++)
                for (int e = 0; e < d; e++) out[(size_t)qh * d + e] = 0.0;
            continue;
        }
        const float **kr = (const float **)malloc(sizeof(float *) * n);
        const float **vr = (const float **)malloc(sizeof(float *) * n);
        double *sc = (double *)malloc(sizeof(double) * n);
        if (!kr || !vr || !sc) { free(kr); free(vr); free(sc); return ORC_ERR_NOMEM; }
        int64_t c = 0;
        for (int64_t i = 0; i < H->glen; i++, c++) { kr[c] = H->gk + i * d; vr[c] = H->gv + i * d; }
        for (int s = 0; s < W; s++)
            if (H->ring_pos[s] >= 0) { kr[c] = H->ring_k + (size_t)s * d; vr[c] = H->ring_v + (size_t)s * d; c++; }
        for (int qh = h * G; qh < (h + 1) * G; qh++)
            softmax_av(q + (size_t)qh * d, kr, vr, n, d, scale, sc, out + (size_t)qh * d);
        free(kr); free(vr); free(sc);
    }
    return ORC_OK;
}

/* The same for several sequences at once (one decode step of one layer);
 * independent (sequence, kv head) units run on separate host threads and
 * nothing else is parallel.  q/out: [n_seqs][n_q_heads][d]. */
int orc_attend_cached_batch(const orc_state *S, int layer, int n_seqs, const int32_t *seq_ids,
                            const float *q, double scale, double *out, int *threads_used) {
    if (!S || !S->c.keep_payload) return ORC_ERR_ARG;
    const int Hq = S->c.n_q_heads, Hk = S->c.n_kv_heads, d = S->c.head_dim, W = S->c.w_local;
    const int G = Hq / Hk;
    int rc_all = ORC_OK, nthr = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        nthr = omp_get_num_threads();
    }
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int u = 0; u < n_seqs * Hk; u++) {
        const int b = u / Hk, h = u % Hk;
        const orc_head *H = &S->sl[(size_t)seq_ids[b] * S->c.n_layers + layer].h[h];
        int64_t n = H->glen;
        for (int s = 0; s < W; s++) if (H->ring_pos[s] >= 0) n++;
        double *o = out + ((size_t)b * Hq + (size_t)h * G) * d;
        if (n == 0) { for (int e = 0; e < G * d; e++) o[e] = 0.0; continue; }
        const float **kr = (const float **)malloc(sizeof(float *) * n);
        const float **vr = (const float **)malloc(sizeof(float *) * n);
        double *sc = (double *)malloc(sizeof(double) * n);
        if (!kr || !vr || !sc) { free(kr); free(vr); free(sc); rc_all = ORC_ERR_NOMEM; continue; }
        int64_t c = 0;
        for (int64_t i = 0; i < H->glen; i++, c++) { kr[c] = H->gk + i * d; vr[c] = H->gv + i * d; }
        for (int s = 0; s < W; s++)
            if (H->ring_pos[s] >= 0) { kr[c] = H->ring_k + (size_t)s * d; vr[c] = H->ring_v + (size_t)s * d; c++; }
        for (int j = 0; j < G; j++)
            softmax_av(q + ((size_t)b * Hq + (size_t)h * G + j) * d, kr, vr, n, d, scale, sc, o + (size_t)j * d);
        free(kr); free(vr); free(sc);
    }
    if (threads_used) *threads_used = nthr;
    return rc_all;
}

/*
 * Definition attention (Sec. 4.2 mask equation on Sec. 2.1 attention) from the
 * full history of ONE sequence/layer:
 *   K, V : [n_hist][n_kv_heads][d]     g : [n_hist][n_kv_heads]
 *   q    : [n_q][n_q_heads][d]         q_pos[n_q] : position i of each query
 * Key j is visible to query i iff j <= i and (i - j < W  or  g_j >= tau).
 * out: [n_q][n_q_heads][d] doubles.
 */
int orc_attend_definition(int n_q_heads, int n_kv_heads, int d, int w_local, float tau,
                          double scale, int64_t n_hist, const float *K, const float *V,
                          const float *g, int64_t n_q, const float *q, const int64_t *q_pos,
                          double *out) {
    if (n_q_heads % n_kv_heads) return ORC_ERR_ARG;
    const int G = n_q_heads / n_kv_heads;
    int rc_all = ORC_OK;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int64_t r = 0; r < n_q; r++) {
        const int64_t i = q_pos[r];
        if (i < 0 || i >= n_hist) { rc_all = ORC_ERR_ARG; continue; }
        const float **kr = (const float **)malloc(sizeof(float *) * (size_t)(i + 1));
        const float **vr = (const float **)malloc(sizeof(float *) * (size_t)(i + 1));
        double *sc = (double *)malloc(sizeof(double) * (size_t)(i + 1));
        if (!kr || !vr || !sc) { free(kr); free(vr); free(sc); rc_all = ORC_ERR_NOMEM; continue; }
        for (int h = 0; h < n_kv_heads; h++) {
            int64_t n = 0;
            for (int64_t j = 0; j <= i; j++) {
                size_t row = (size_t)j * n_kv_heads + h;
                if ((i - j < w_local) || (g[row] >= tau)) {
                    kr[n] = K + row * d; vr[n] = V + row * d; n++;
                }
            }
            for (int jq = 0; jq < G; jq++) {
                size_t qh = (size_t)h * G + jq;
                softmax_av(q + ((size_t)r * n_q_heads + qh) * d, kr, vr, n, d, scale, sc,
                           out + ((size_t)r * n_q_heads + qh) * d);
            }
        }
        free(kr); free(vr); free(sc);
    }
    return rc_all;
}

/*
 * Training-time soft form of the same attention (Sec. 3.2, "Write-Gated
 * Attention" equation): weights exp(s_ij) * m_ij with
 * m_ij = max(1(i-j < W), g_j); with eps >= 0 the log-space form
 * exp(s_ij + log(m_ij + eps)) is used instead when use_log != 0.
 * With binary g it must reproduce orc_attend_definition; kept only as a
 * cross-check of the mask code.
 */
int orc_attend_soft(int n_q_heads, int n_kv_heads, int d, int w_local, double scale,
                    int64_t n_hist, const float *K, const float *V, const float *g,
                    int64_t n_q, const float *q, const int64_t *q_pos, int use_log, double eps,
                    double *out) {
    if (n_q_heads % n_kv_heads) return ORC_ERR_ARG;
    const int G = n_q_heads / n_kv_heads;
    for (int64_t r = 0; r < n_q; r++) {
        const int64_t i = q_pos[r];
        if (i < 0 || i >= n_hist) return ORC_ERR_ARG;
        double *sc = (double *)malloc(sizeof(double) * (size_t)(i + 1));
        if (!sc) return ORC_ERR_NOMEM;
        for (int qh = 0; qh < n_q_heads; qh++) {
            const int h = qh / G;
            const float *qv = q + ((size_t)r * n_q_heads + qh) * d;
            double mx = -INFINITY;
            for (int64_t j = 0; j <= i; j++) {
                size_t row = (size_t)j * n_kv_heads + h;
                double s = 0.0;
                for (int e = 0; e < d; e++) s += (double)qv[e] * (double)K[row * d + e];
                s *= scale;
                double m = (i - j < w_local) ? 1.0 : 0.0;
                if ((double)g[row] > m) m = (double)g[row];
                if (use_log) { s += log(m + eps); sc[j] = s; }
                else sc[j] = s; /* weight applied below */
                if (s > mx && (use_log || m > 0.0)) mx = s;
            }
            double den = 0.0;
            double *o = out + ((size_t)r * n_q_heads + qh) * d;
            for (int e = 0; e < d; e++) o[e] = 0.0;
            for (int64_t j = 0; j <= i; j++) {
                size_t row = (size_t)j * n_kv_heads + h;
                double w = exp(sc[j] - mx);
                if (!use_log) {
                    double m = (i - j < w_local) ? 1.0 : 0.0;
                    if ((double)g[row] > m) m = (double)g[row];
                    w *= m;
                }
                sc[j] = w;
                den += w;
            }
            for (int64_t j = 0; j <= i; j++) {
                size_t row = (size_t)j * n_kv_heads + h;
                double w = sc[j] / den;
                for (int e = 0; e < d; e++) o[e] += w * (double)V[row * d + e];
            }
        }
        free(sc);
    }
    return ORC_OK;
}

/*
 * Linear write gate used by the chunked-prefill workload: one weight vector
 * per kv head on the layer's hidden state, g = sigmoid(w_h . x_t), i.e. the
 * Sec. 3.2 gate equation with the hidden layer removed.
 *   hidden: [T][dim], w: [n_kv_heads][dim]; logit_out, g_out: [T][n_kv_heads].
 */
int orc_linear_gate(int64_t T, int dim, int n_kv_heads, const float *hidden, const float *w,
                    double *logit_out, double *g_out) {
    /* tokens are independent: spread them over the host threads */
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; t++)
        for (int h = 0; h < n_kv_heads; h++) {
            double s = 0.0;
            for (int e = 0; e < dim; e++) s += (double)hidden[t * dim + e] * (double)w[(size_t)h * dim + e];
            if (logit_out) logit_out[t * n_kv_heads + h] = s;
            if (g_out) g_out[t * n_kv_heads + h] = 1.0 / (1.0 + exp(-s));
        }
    return ORC_OK;
}

/*
 * Budgeted eviction on the global cache (appendix "Eviction policy implementation").
 *
 * Importance of the N entries of one head's global cache, from the queries of the
 * last n_obs positions (the observation window), in the appendix' three steps:
 *   (1) A^(hq) = Softmax(Q_obs^(hq) K^T * scale) for every query head hq of the group,
 *   (2) S_raw_j = sum_i max_hq A^(hq)_ij,
 *   (3) S = MaxPool(S_raw, pool_w) along the cache order.
 * Readings: K is the head's global cache alone (the only entries that can be evicted;
 * every one of them is older than the window, so every observation query sees all of
 * them and no mask is needed) and the softmax is normalised over these N entries;
 * the pooling window is centred (j - pool_w/2 .. j + pool_w/2) and clipped at the
 * ends of the cache, pool_w odd.
 *   q_obs : [n_obs][n_q_heads][d]; s_raw_out, s_out : [N] (either may be NULL)
 */
int orc_evict_scores(const orc_state *S, int layer, int seq, int h, const float *q_obs, int n_obs,
                     double scale, int pool_w, double *s_raw_out, double *s_out) {
    if (!S || !S->c.keep_payload || layer < 0 || layer >= S->c.n_layers || seq < 0 ||
        seq >= S->c.max_seqs || h < 0 || h >= S->c.n_kv_heads || n_obs < 1 || pool_w < 1 ||
        pool_w % 2 == 0 || !q_obs)
        return ORC_ERR_ARG;
    const orc_head *H = &S->sl[(size_t)seq * S->c.n_layers + layer].h[h];
    const int d = S->c.head_dim, G = S->c.n_q_heads / S->c.n_kv_heads;
    const int64_t N = H->glen;
    if (N == 0) return ORC_OK;
    double *raw = (double *)calloc((size_t)N, sizeof(double));
    double *a = (double *)malloc(sizeof(double) * (size_t)N * G);
    if (!raw || !a) { free(raw); free(a); return ORC_ERR_NOMEM; }
    for (int i = 0; i < n_obs; i++) {
        for (int g = 0; g < G; g++) {
            const float *q = q_obs + ((size_t)i * S->c.n_q_heads + (size_t)h * G + g) * d;
            double *row = a + (size_t)g * N;
            double mx = -INFINITY;
            for (int64_t j = 0; j < N; j++) {
                double dot = 0.0;
                for (int e = 0; e < d; e++) dot += (double)q[e] * (double)H->gk[j * d + e];
                row[j] = dot * scale;
                if (row[j] > mx) mx = row[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j < N; j++) { row[j] = exp(row[j] - mx); den += row[j]; }
            for (int64_t j = 0; j < N; j++) row[j] /= den;
        }
        for (int64_t j = 0; j < N; j++) {
            double best = a[j];
            for (int g = 1; g < G; g++) if (a[(size_t)g * N + j] > best) best = a[(size_t)g * N + j];
            raw[j] += best;
        }
    }
    for (int64_t j = 0; j < N; j++) {
        if (s_raw_out) s_raw_out[j] = raw[j];
        if (s_out) {
            double best = raw[j];
            for (int64_t jj = j - pool_w / 2; jj <= j + pool_w / 2; jj++)
                if (jj >= 0 && jj < N && raw[jj] > best) best = raw[jj];
            s_out[j] = best;
        }
    }
    free(raw); free(a);
    return ORC_OK;
}

/* Order of fp32 scores used for eviction: the total order of the bit patterns
 * (negative < positive, NaN with the sign bit clear above everything). */
static uint32_t score_key(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

/*
 * Removes, from every head of the given sequences, the floor(frac * N) entries of its
 * global cache with the lowest scores ("remove the bottom 10 %" in the appendix; the
 * policy works on each kv head on its own).  Among equal scores the older entry goes
 * first.  The survivors keep their order and are packed to the front; pages that no
 * longer hold an entry go back to the free stack, units in (position in the call, kv
 * head) order, a unit's pages in ascending table index.  The page order is this
 * project's own rule (the paper has none).
 *   scores : float [n_seqs * n_kv_heads][stride], entry j of unit (b, h) at
 *            scores[(b * n_kv_heads + h) * stride + j]
 *   n_evicted_out (optional): [n_seqs * n_kv_heads]
 */
int orc_evict_apply(orc_state *S, int layer, int n_seqs, const int32_t *seq_ids, const float *scores,
                    int64_t stride, float frac, int64_t *n_evicted_out) {
    if (!S || layer < 0 || layer >= S->c.n_layers || n_seqs < 0 || !seq_ids || !scores ||
        !(frac >= 0.0f) || !(frac <= 1.0f))
        return ORC_ERR_ARG;
    const int Hk = S->c.n_kv_heads, d = S->c.head_dim, P = S->c.page_size;
    for (int b = 0; b < n_seqs; b++) {
        if (seq_ids[b] < 0 || seq_ids[b] >= S->c.max_seqs) return ORC_ERR_ARG;
        for (int b2 = 0; b2 < b; b2++) if (seq_ids[b2] == seq_ids[b]) return ORC_ERR_ARG;
    }
    for (int b = 0; b < n_seqs; b++)
        for (int h = 0; h < Hk; h++) {
            orc_head *H = &S->sl[(size_t)seq_ids[b] * S->c.n_layers + layer].h[h];
            const float *sc = scores + ((size_t)b * Hk + h) * stride;
            const int64_t N = H->glen;
            if (N > stride) return ORC_ERR_ARG;
            const int64_t n_e = (int64_t)floor((double)frac * (double)N);
            if (n_evicted_out) n_evicted_out[(size_t)b * Hk + h] = n_e;
            if (n_e == 0) continue;
            /* plain selection: n_e times take the smallest (key, index) not yet taken */
            char *gone = (char *)calloc((size_t)N, 1);
            if (!gone) return ORC_ERR_NOMEM;
            for (int64_t r = 0; r < n_e; r++) {
                int64_t best = -1;
                for (int64_t j = 0; j < N; j++)
                    if (!gone[j] && (best < 0 || score_key(sc[j]) < score_key(sc[best]))) best = j;
                gone[best] = 1;
            }
            int64_t w = 0;
            for (int64_t j = 0; j < N; j++) {
                if (gone[j]) continue;
                if (w != j) {
                    H->gpos[w] = H->gpos[j];
                    if (S->c.keep_payload) {
                        memmove(H->gk + w * d, H->gk + j * d, sizeof(float) * d);
                        memmove(H->gv + w * d, H->gv + j * d, sizeof(float) * d);
                    }
                }
                w++;
            }
            free(gone);
            const int64_t old_pages = (N + P - 1) / P, new_pages = (w + P - 1) / P;
            for (int64_t lp = new_pages; lp < old_pages; lp++) {
                S->free_stack[S->free_top++] = H->global_pt[lp];
                H->global_pt[lp] = -1;
            }
            H->glen = w;
        }
    return ORC_OK;
}

/*
 * Read-time page selection over the admitted cache (appendix "Synergy with KV
 * Selection": Quest-style selection with key landmarks, the per-page minimum and
 * maximum key vectors, at a budget of so many KVs per query).  The paper only names
 * the method; the steps below are the published Quest procedure in the form this
 * project reads it for grouped-query attention:
 *   landmarks of page p of a head's global cache: lo_p[e] = min, hi_p[e] = max of
 *     K_j[e] over the entries j the page holds (the last page may be partly filled);
 *   criticality of the page for a decode query:
 *     U_p = max over the query heads g of the group of sum_e max(q_g[e] lo_p[e], q_g[e] hi_p[e]),
 *     an upper bound of every q_g . K_j in the page; one selection per kv head, since
 *     the group shares the pages;
 *   the min(n_pages, budget_pages) pages with the largest U are read, together with
 *     the local window, which is always read.
 *   q : [n_q_heads][d]; u_out : [ceil(N/P)] for head h.
 */
int orc_quest_page_scores(const orc_state *S, int layer, int seq, int h, const float *q, double *u_out) {
    if (!S || !S->c.keep_payload || layer < 0 || layer >= S->c.n_layers || seq < 0 ||
        seq >= S->c.max_seqs || h < 0 || h >= S->c.n_kv_heads || !q || !u_out)
        return ORC_ERR_ARG;
    const orc_head *H = &S->sl[(size_t)seq * S->c.n_layers + layer].h[h];
    const int d = S->c.head_dim, P = S->c.page_size, G = S->c.n_q_heads / S->c.n_kv_heads;
    const int64_t N = H->glen, n_pages = (N + P - 1) / P;
    for (int64_t p = 0; p < n_pages; p++) {
        const int64_t j0 = p * P, j1 = (j0 + P < N) ? j0 + P : N;
        double best = -INFINITY;
        for (int g = 0; g < G; g++) {
            const float *qg = q + ((size_t)h * G + g) * d;
            double sum = 0.0;
            for (int e = 0; e < d; e++) {
                double lo = (double)H->gk[j0 * d + e], hi = lo;
                for (int64_t j = j0 + 1; j < j1; j++) {
                    const double x = (double)H->gk[j * d + e];
                    if (x < lo) lo = x;
                    if (x > hi) hi = x;
                }
                const double a = (double)qg[e] * lo, b = (double)qg[e] * hi;
                sum += a > b ? a : b;
            }
            if (sum > best) best = sum;
        }
        u_out[p] = best;
    }
    return ORC_OK;
}

/* The pages to read: the n_sel = min(n_pages, budget_pages) largest scores in the total
 * order of the fp32 bit patterns, among equal scores the page with the lower index
 * first; returned as ascending page indices.  sel_out: [budget_pages]. */
int orc_quest_select(const float *scores, int64_t n_pages, int64_t budget_pages, int32_t *sel_out,
                     int32_t *n_sel_out) {
    if (!scores || n_pages < 0 || budget_pages < 0 || !sel_out || !n_sel_out) return ORC_ERR_ARG;
    const int64_t n_sel = n_pages < budget_pages ? n_pages : budget_pages;
    char *taken = (char *)calloc((size_t)(n_pages > 0 ? n_pages : 1), 1);
    if (!taken) return ORC_ERR_NOMEM;
    for (int64_t r = 0; r < n_sel; r++) {
        int64_t best = -1;
        for (int64_t p = 0; p < n_pages; p++)
            if (!taken[p] && (best < 0 || score_key(scores[p]) > score_key(scores[best]))) best = p;
        taken[best] = 1;
    }
    int64_t w = 0;
    for (int64_t p = 0; p < n_pages; p++) if (taken[p]) sel_out[w++] = (int32_t)p;
    *n_sel_out = (int32_t)n_sel;
    free(taken);
    return ORC_OK;
}

/* Decode attention of one sequence/layer over the local window and, per kv head, only the
 * selected pages of its global cache.  sel: [n_kv_heads][stride] ascending page indices,
 * n_sel: [n_kv_heads].  q, out: [n_q_heads][d]. */
int orc_attend_selected(const orc_state *S, int seq, int layer, const float *q, const int32_t *sel,
                        const int32_t *n_sel, int64_t stride, double scale, double *out) {
    if (!S || !S->c.keep_payload || !q || !sel || !n_sel || !out) return ORC_ERR_ARG;
    const int Hq = S->c.n_q_heads, Hk = S->c.n_kv_heads, d = S->c.head_dim, W = S->c.w_local;
    const int G = Hq / Hk, P = S->c.page_size;
    const orc_sl *sl = &S->sl[(size_t)seq * S->c.n_layers + layer];
    for (int h = 0; h < Hk; h++) {
        const orc_head *H = &sl->h[h];
        const int64_t n_pages = (H->glen + P - 1) / P;
        int64_t n = 0;
        for (int i = 0; i < n_sel[h]; i++) {
            const int64_t p = sel[(size_t)h * stride + i];
            if (p < 0 || p >= n_pages || (i > 0 && p <= sel[(size_t)h * stride + i - 1])) return ORC_ERR_ARG;
            n += ((p + 1) * P <= H->glen) ? P : H->glen - p * P;
        }
        for (int s = 0; s < W; s++) if (H->ring_pos[s] >= 0) n++;
        if (n == 0) {
            for (int qh = h * G; qh < (h + 1) * G; qh++)
                for (int e = 0; e < d; e++) out[(size_t)qh * d + e] = 0.0;
            continue;
        }
        const float **kr = (const float **)malloc(sizeof(float *) * n);
        const float **vr = (const float **)malloc(sizeof(float *) * n);
        double *sc = (double *)malloc(sizeof(double) * n);
        if (!kr || !vr || !sc) { free(kr); free(vr); free(sc); return ORC_ERR_NOMEM; }
        int64_t c = 0;
        for (int i = 0; i < n_sel[h]; i++) {
            const int64_t p = sel[(size_t)h * stride + i];
            for (int64_t j = p * P; j < (p + 1) * P && j < H->glen; j++, c++) { kr[c] = H->gk + j * d; vr[c] = H->gv + j * d; }
        }
        for (int s = 0; s < W; s++)
            if (H->ring_pos[s] >= 0) { kr[c] = H->ring_k + (size_t)s * d; vr[c] = H->ring_v + (size_t)s * d; c++; }
        for (int qh = h * G; qh < (h + 1) * G; qh++)
            softmax_av(q + (size_t)qh * d, kr, vr, n, d, scale, sc, out + (size_t)qh * d);
        free(kr); free(vr); free(sc);
    }
    return ORC_OK;
}

/* Round a double to the nearest bfloat16 (ties to even) and return it as a double.
 * Finite inputs in the normal float range only (that is all the callers produce). */
static double round_to_bf16(double x) {
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/*
 * Write-Gate MLP (Sec. 3.2, feature equation and gate equation).  Per token t and
 * kv head h:
 *     x = [ RMSNorm(k[t][h]) ; RMSNorm(k_rope[t][h]) ]                 (2d numbers)
 *     g = sigmoid( W2[h] . GELU( W1[h] x + b1[h] ) + b2[h] )
 * The paper leaves the hidden width, the GELU flavour and the RMSNorm constants
 * open; here the width is an argument, GELU is the exact one,
 * GELU(z) = z/2 (1 + erf(z / sqrt 2)), and RMSNorm(v) = v / sqrt(mean(v^2) + eps)
 * carries no learnable scale.
 *   k, k_rope : [T][H][d]      W1 : [H][width][2d]    b1 : [H][width]
 *   W2        : [H][width]     b2 : [H]               logit_out, g_out : [T][H]
 * feature_bf16 != 0 rounds every normalised feature to bfloat16 before the first
 * product, as a bf16 model that hands its RMSNorm output to a bf16 matmul does.
 */
int orc_gate_mlp(int64_t T, int H, int d, int width, const float *k, const float *k_rope,
                 const float *W1, const float *b1, const float *W2, const float *b2, double eps,
                 int feature_bf16, double *logit_out, double *g_out) {
    if (T < 0 || H < 1 || d < 1 || width < 1) return ORC_ERR_ARG;
    int rc_all = ORC_OK;
    /* tokens are independent: spread them over the host threads */
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; t++) {
        double *x = (double *)malloc(sizeof(double) * 2 * (size_t)d);
        if (!x) {
#pragma omp atomic write
            rc_all = ORC_ERR_NOMEM;
            continue;
        }
        for (int h = 0; h < H; h++) {
            for (int part = 0; part < 2; part++) {
                const float *v = (part == 0 ? k : k_rope) + ((size_t)t * H + h) * d;
                double ss = 0.0;
                for (int e = 0; e < d; e++) ss += (double)v[e] * (double)v[e];
                const double r = 1.0 / sqrt(ss / d + eps);
                for (int e = 0; e < d; e++) {
                    const double xn = (double)v[e] * r;
                    x[part * d + e] = feature_bf16 ? round_to_bf16(xn) : xn;
                }
            }
            double logit = (double)b2[h];
            for (int u = 0; u < width; u++) {
                const float *w = W1 + ((size_t)h * width + u) * 2 * d;
                double z = (double)b1[(size_t)h * width + u];
                for (int e = 0; e < 2 * d; e++) z += (double)w[e] * x[e];
                const double gelu = 0.5 * z * (1.0 + erf(z / sqrt(2.0)));
                logit += (double)W2[(size_t)h * width + u] * gelu;
            }
            if (logit_out) logit_out[t * H + h] = logit;
            if (g_out) g_out[t * H + h] = 1.0 / (1.0 + exp(-logit));
        }
        free(x);
    }
    return rc_all;
}


/*
 * Training-time Write-Gated Attention of a whole sequence (Sec. 3.2): causal softmax of
 *   s_ij = scale * q_i . k_j + log(m_ij + eps),   m_ij = max(1(i - j < W), g_j),
 * the log-space form of weighting exp(q_i . k_j * scale) by m_ij ("Log-space transformation
 * for efficient training", with the small eps the text adds inside the logarithm).
 *   Q: [T][Hq][d]   K, V: [T][Hkv][d]   g: [T][Hkv]; query head qh reads kv head qh / (Hq/Hkv).
 *   out: [T][Hq][d], lse: [T][Hq] = log sum_j exp(s_ij) (natural logarithm); either may be NULL.
 */
int orc_soft_attn_forward(int64_t T, int Hq, int Hkv, int d, int W, double scale, double eps,
                          const float *Q, const float *K, const float *V, const float *g,
                          double *out, double *lse) {
    if (T < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || W < 1) return ORC_ERR_ARG;
    const int G = Hq / Hkv;
    int rc_all = ORC_OK;
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t i = 0; i < T; i++) {
        double *s = (double *)malloc(sizeof(double) * (size_t)(i + 1));
        if (!s) { rc_all = ORC_ERR_NOMEM; continue; }
        for (int qh = 0; qh < Hq; qh++) {
            const int h = qh / G;
            const float *qi = Q + ((size_t)i * Hq + qh) * d;
            double mx = -INFINITY;
            for (int64_t j = 0; j <= i; j++) {
                const size_t row = (size_t)j * Hkv + h;
                double dot = 0.0;
                for (int e = 0; e < d; e++) dot += (double)qi[e] * (double)K[row * d + e];
                double m = (i - j < W) ? 1.0 : 0.0;
                if ((double)g[row] > m) m = (double)g[row];
                s[j] = scale * dot + log(m + eps);
                if (s[j] > mx) mx = s[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j <= i; j++) den += exp(s[j] - mx);
            const double l = mx + log(den);
            if (lse) lse[(size_t)i * Hq + qh] = l;
            if (out) {
                double *o = out + ((size_t)i * Hq + qh) * d;
                for (int e = 0; e < d; e++) o[e] = 0.0;
                for (int64_t j = 0; j <= i; j++) {
                    const double p = exp(s[j] - l);
                    const float *vj = V + ((size_t)j * Hkv + h) * d;
                    for (int e = 0; e < d; e++) o[e] += p * (double)vj[e];
                }
            }
        }
        free(s);
    }
    return rc_all;
}

/*
 * Gradients of a scalar loss through orc_soft_attn_forward, given dO = dLoss/dOut [T][Hq][d].
 * With p_ij = exp(s_ij - lse_i), o_i = sum_j p_ij v_j:
 *   dV_j  = sum_i p_ij dO_i
 *   dS_ij = p_ij (dO_i . v_j - dO_i . o_i)          (derivative with respect to s_ij)
 *   dQ_i  = scale sum_j dS_ij k_j      dK_j = scale sum_i dS_ij q_i
 *   dg_j  = sum_i dS_ij * d log(m_ij + eps)/dg_j = sum_{i : g_j > 1(i-j<W)} dS_ij / (g_j + eps)
 * (m_ij follows g_j only where g_j exceeds the window indicator).  A kv head collects the terms
 * of all query heads of its group.  dQ: [T][Hq][d], dK, dV: [T][Hkv][d], dg: [T][Hkv].
 */
int orc_soft_attn_backward(int64_t T, int Hq, int Hkv, int d, int W, double scale, double eps,
                           const float *Q, const float *K, const float *V, const float *g,
                           const float *dO, double *dQ, double *dK, double *dV, double *dg) {
    if (T < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || W < 1) return ORC_ERR_ARG;
    const int G = Hq / Hkv;
    int rc_all = ORC_OK;
    for (size_t x = 0; x < (size_t)T * Hq * d; x++) dQ[x] = 0.0;
    for (size_t x = 0; x < (size_t)T * Hkv * d; x++) { dK[x] = 0.0; dV[x] = 0.0; }
    for (size_t x = 0; x < (size_t)T * Hkv; x++) dg[x] = 0.0;
    /* a kv head owns its rows of dK, dV, dg: one thread per kv head, no shared sums */
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < Hkv; h++) {
        double *p = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
        if (!p || !o) { free(p); free(o); rc_all = ORC_ERR_NOMEM; continue; }
        for (int jq = 0; jq < G; jq++) {
            const int qh = h * G + jq;
            for (int64_t i = 0; i < T; i++) {
                const float *qi = Q + ((size_t)i * Hq + qh) * d;
                const float *doi = dO + ((size_t)i * Hq + qh) * d;
                double mx = -INFINITY;
                for (int64_t j = 0; j <= i; j++) {
                    const size_t row = (size_t)j * Hkv + h;
                    double dot = 0.0;
                    for (int e = 0; e < d; e++) dot += (double)qi[e] * (double)K[row * d + e];
                    double m = (i - j < W) ? 1.0 : 0.0;
                    if ((double)g[row] > m) m = (double)g[row];
                    p[j] = scale * dot + log(m + eps);
                    if (p[j] > mx) mx = p[j];
                }
                double den = 0.0;
                for (int64_t j = 0; j <= i; j++) { p[j] = exp(p[j] - mx); den += p[j]; }
                for (int e = 0; e < d; e++) o[e] = 0.0;
                for (int64_t j = 0; j <= i; j++) {
                    p[j] /= den;
                    const float *vj = V + ((size_t)j * Hkv + h) * d;
                    for (int e = 0; e < d; e++) o[e] += p[j] * (double)vj[e];
                }
                double Di = 0.0;
                for (int e = 0; e < d; e++) Di += (double)doi[e] * o[e];
                double *dqi = dQ + ((size_t)i * Hq + qh) * d;
                for (int64_t j = 0; j <= i; j++) {
                    const size_t row = (size_t)j * Hkv + h;
                    const float *kj = K + row * d, *vj = V + row * d;
                    double dP = 0.0;
                    for (int e = 0; e < d; e++) dP += (double)doi[e] * (double)vj[e];
                    const double dS = p[j] * (dP - Di);
                    for (int e = 0; e < d; e++) {
                        dV[row * d + e] += p[j] * (double)doi[e];
                        dqi[e] += scale * dS * (double)kj[e];
                        dK[row * d + e] += scale * dS * (double)qi[e];
                    }
                    const double ind = (i - j < W) ? 1.0 : 0.0;
                    if ((double)g[row] > ind) dg[row] += dS / ((double)g[row] + eps);
                }
            }
        }
        free(p); free(o);
    }
    return rc_all;
}

/*
 * The same gradients for a sample of the outputs, for sequences too long for the full
 * function: dQ of the query rows listed in `rows` (all query heads), and dK, dV, dg of the
 * keys j >= j_first of kv head h (a tail of the sequence: only the queries i >= j see them,
 * and each such query still needs its whole row of weights for lse_i and dO_i . o_i).
 *   dQ_rows: [n_rows][Hq][d]   dK_tail, dV_tail: [T - j_first][d]   dg_tail: [T - j_first]
 */
int orc_soft_attn_backward_sampled(int64_t T, int Hq, int Hkv, int d, int W, double scale, double eps,
                                   const float *Q, const float *K, const float *V, const float *g,
                                   const float *dO, int64_t n_rows, const int64_t *rows, double *dQ_rows,
                                   int h, int64_t j_first, double *dK_tail, double *dV_tail, double *dg_tail) {
    if (T < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || W < 1 || h < 0 || h >= Hkv || j_first < 0 || j_first > T)
        return ORC_ERR_ARG;
    const int G = Hq / Hkv;
    int rc_all = ORC_OK;
    /* ---- dQ of the sampled rows ---- */
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; r++) {
        const int64_t i = rows[r];
        if (i < 0 || i >= T) { rc_all = ORC_ERR_ARG; continue; }
        double *p = (double *)malloc(sizeof(double) * (size_t)(i + 1));
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
        if (!p || !o) { free(p); free(o); rc_all = ORC_ERR_NOMEM; continue; }
        for (int qh = 0; qh < Hq; qh++) {
            const int hh = qh / G;
            const float *qi = Q + ((size_t)i * Hq + qh) * d, *doi = dO + ((size_t)i * Hq + qh) * d;
            double mx = -INFINITY;
            for (int64_t j = 0; j <= i; j++) {
                const size_t row = (size_t)j * Hkv + hh;
                double dot = 0.0;
                for (int e = 0; e < d; e++) dot += (double)qi[e] * (double)K[row * d + e];
                double m = (i - j < W) ? 1.0 : 0.0;
                if ((double)g[row] > m) m = (double)g[row];
                p[j] = scale * dot + log(m + eps);
                if (p[j] > mx) mx = p[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j <= i; j++) { p[j] = exp(p[j] - mx); den += p[j]; }
            for (int e = 0; e < d; e++) o[e] = 0.0;
            for (int64_t j = 0; j <= i; j++) {
                p[j] /= den;
                const float *vj = V + ((size_t)j * Hkv + hh) * d;
                for (int e = 0; e < d; e++) o[e] += p[j] * (double)vj[e];
            }
            double Di = 0.0;
            for (int e = 0; e < d; e++) Di += (double)doi[e] * o[e];
            double *dq = dQ_rows + ((size_t)r * Hq + qh) * d;
            for (int e = 0; e < d; e++) dq[e] = 0.0;
            for (int64_t j = 0; j <= i; j++) {
                const size_t row = (size_t)j * Hkv + hh;
                double dP = 0.0;
                for (int e = 0; e < d; e++) dP += (double)doi[e] * (double)V[row * d + e];
                const double dS = p[j] * (dP - Di);
                for (int e = 0; e < d; e++) dq[e] += scale * dS * (double)K[row * d + e];
            }
        }
        free(p); free(o);
    }
    /* ---- dK, dV, dg of the tail keys of kv head h ---- */
    const int64_t n = T - j_first;
    for (size_t x = 0; x < (size_t)n * d; x++) { dK_tail[x] = 0.0; dV_tail[x] = 0.0; }
    for (int64_t x = 0; x < n; x++) dg_tail[x] = 0.0;
    if (n == 0) return rc_all;
    double *PS = (double *)malloc(sizeof(double) * (size_t)n * (size_t)n);
    double *DS = (double *)malloc(sizeof(double) * (size_t)n * (size_t)n);
    if (!PS || !DS) { free(PS); free(DS); return ORC_ERR_NOMEM; }
    for (int jq = 0; jq < G; jq++) {
        const int qh = h * G + jq;
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t i = j_first; i < T; i++) {
            double *p = (double *)malloc(sizeof(double) * (size_t)(i + 1));
            double *o = (double *)malloc(sizeof(double) * (size_t)d);
            if (!p || !o) { free(p); free(o); rc_all = ORC_ERR_NOMEM; continue; }
            const float *qi = Q + ((size_t)i * Hq + qh) * d, *doi = dO + ((size_t)i * Hq + qh) * d;
            double mx = -INFINITY;
            for (int64_t j = 0; j <= i; j++) {
                const size_t row = (size_t)j * Hkv + h;
                double dot = 0.0;
                for (int e = 0; e < d; e++) dot += (double)qi[e] * (double)K[row * d + e];
                double m = (i - j < W) ? 1.0 : 0.0;
                if ((double)g[row] > m) m = (double)g[row];
                p[j] = scale * dot + log(m + eps);
                if (p[j] > mx) mx = p[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j <= i; j++) { p[j] = exp(p[j] - mx); den += p[j]; }
            for (int e = 0; e < d; e++) o[e] = 0.0;
            for (int64_t j = 0; j <= i; j++) {
                p[j] /= den;
                const float *vj = V + ((size_t)j * Hkv + h) * d;
                for (int e = 0; e < d; e++) o[e] += p[j] * (double)vj[e];
            }
            double Di = 0.0;
            for (int e = 0; e < d; e++) Di += (double)doi[e] * o[e];
            for (int64_t j = j_first; j <= i; j++) {
                const float *vj = V + ((size_t)j * Hkv + h) * d;
                double dP = 0.0;
                for (int e = 0; e < d; e++) dP += (double)doi[e] * (double)vj[e];
                PS[(size_t)(i - j_first) * n + (j - j_first)] = p[j];
                DS[(size_t)(i - j_first) * n + (j - j_first)] = p[j] * (dP - Di);
            }
            free(p); free(o);
        }
        for (int64_t i = j_first; i < T; i++) {
            const float *qi = Q + ((size_t)i * Hq + qh) * d, *doi = dO + ((size_t)i * Hq + qh) * d;
            for (int64_t j = j_first; j <= i; j++) {
                const size_t row = (size_t)j * Hkv + h;
                const double pij = PS[(size_t)(i - j_first) * n + (j - j_first)];
                const double dS = DS[(size_t)(i - j_first) * n + (j - j_first)];
                double *dk = dK_tail + (size_t)(j - j_first) * d, *dv = dV_tail + (size_t)(j - j_first) * d;
                for (int e = 0; e < d; e++) {
                    dv[e] += pij * (double)doi[e];
                    dk[e] += scale * dS * (double)qi[e];
                }
                const double ind = (i - j < W) ? 1.0 : 0.0;
                if ((double)g[row] > ind) dg_tail[j - j_first] += dS / ((double)g[row] + eps);
            }
        }
    }
    free(PS); free(DS);
    return rc_all;
}

/*
 * Sparsity term of the training objective (Sec. 3.3): the mean over all n scores of
 * g + g (1 - g), and its derivative (2 - 2 g) / n with respect to every score.
 */
int orc_sparsity_loss(int64_t n, const float *g, double *loss, double *dg) {
    if (n < 1) return ORC_ERR_ARG;
    double acc = 0.0;
    for (int64_t x = 0; x < n; x++) {
        const double v = (double)g[x];
        acc += v + v * (1.0 - v);
        if (dg) dg[x] = (2.0 - 2.0 * v) / (double)n;
    }
    *loss = acc / (double)n;
    return ORC_OK;
}
