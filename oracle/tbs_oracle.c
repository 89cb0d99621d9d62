/*
 * CPU oracle for token-wise RNN-T beam search.  TEST INFRASTRUCTURE ONLY:
 * see tbs_oracle.h.  fp64 throughout, explicit tables, no blocking, no fusion.
 *
 * Readings of the paper taken here where its text leaves a choice:
 *  - Eq. 3 is used as printed: Bl(U,t1,t2) multiplies the blank probabilities
 *    of frames t1 .. t2-1, so Bl(.,t1,S+1) includes the blank that leaves the
 *    last frame of the segment (Eq. 7).
 *  - Eq. 4 allows t1 == t2 (Bl = 1 there): a transducer may emit several
 *    tokens in one frame (Section 3.1).
 *  - A last segment shorter than S is decoded with its true length.
 *  - d is reset to (s,0,...,0) only when a segment starts; afterwards a
 *    hypothesis carries the d it was created with (Eq. 5 of the previous
 *    round, Section 3.2).
 *  - Softmax runs over all V outputs including blank.
 *  - ChooseNthScore is evaluated only when B holds at least N hypotheses;
 *    otherwise the first clause of the test in Algorithm 1 decides.
 *  - The comparison with the threshold is strict, as printed.
 *  - ChooseNBestExpansions ranks all (hypothesis, token) pairs jointly and
 *    leaves blank out.
 *  - Ties: higher score first; equal scores by hypothesis index then token
 *    for expansions, by order of insertion for hypothesis lists.
 *  - On a merge the earlier entry keeps its predictor state (equal tokens
 *    give equal states).
 *  - An expansion of probability exactly zero is not a hypothesis.
 */
#include "tbs_oracle.h"

#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* A value other than zero plants one known mistake (tests use this to show
 * that the pins notice it).  Never set outside tests. */
static int g_mutant = 0;
void orc_set_mutant(int m) { g_mutant = m; }

/* ================================================================== */
/* Score algebra                                                       */
/* ================================================================== */

void orc_softmax(const double *logits, int rows, int V, double *J) {
    for (int r = 0; r < rows; ++r) {
        const double *l = logits + (size_t)r * V;
        double *out = J + (size_t)r * V;
        double mx = l[0];
        for (int k = 1; k < V; ++k)
            if (l[k] > mx) mx = l[k];
        double z = 0.0;
        for (int k = 0; k < V; ++k) {
            out[k] = exp(l[k] - mx);
            z += out[k];
        }
        for (int k = 0; k < V; ++k) out[k] /= z;
    }
}

void orc_blank_product(const double *J, int H, int S, int V, int blank, double *Bl) {
    const int W = S + 1;
    for (int h = 0; h < H; ++h) {
        for (int t1 = 1; t1 <= S + 1; ++t1) {
            for (int t2 = 1; t2 <= S + 1; ++t2) {
                double v;
                if (t1 > t2) {
                    v = 0.0;
                } else if (t1 == t2) {
                    v = 1.0;
                } else {
                    v = 1.0;
                    int last = t2 - 1;
                    if (g_mutant == 1) last = t2 > S ? S : t2; /* planted: off by one frame */
                    for (int tp = t1; tp <= last; ++tp)
                        v *= J[((size_t)h * S + (tp - 1)) * V + blank];
                }
                Bl[((size_t)h * W + (t1 - 1)) * W + (t2 - 1)] = v;
            }
        }
    }
}

void orc_nonblank_expansion_t(const double *J, const double *Bl, const double *d_old,
                              int H, int S, int V, int blank, double *d) {
    const int W = S + 1;
    for (int h = 0; h < H; ++h) {
        for (int k = 0; k < V; ++k) {
            for (int t2 = 1; t2 <= S; ++t2) {
                double acc = 0.0;
                if (k != blank) {
                    for (int t1 = 1; t1 <= S; ++t1) {
                        if (g_mutant == 2 && t1 == t2) continue; /* planted: forbid same-frame emission */
                        /* Eq. 4: one (t1,t2) path family; Eq. 5: sum over t1 */
                        acc += d_old[(size_t)h * S + (t1 - 1)]
                             * Bl[((size_t)h * W + (t1 - 1)) * W + (t2 - 1)]
                             * J[((size_t)h * S + (t2 - 1)) * V + k];
                    }
                }
                d[((size_t)h * V + k) * S + (t2 - 1)] = acc;
            }
        }
    }
}

void orc_nonblank_expansion(const double *d, int H, int S, int V, double *dnb) {
    for (int h = 0; h < H; ++h)
        for (int k = 0; k < V; ++k) {
            double acc = 0.0;
            for (int t2 = 0; t2 < S; ++t2) acc += d[((size_t)h * V + k) * S + t2];
            dnb[(size_t)h * V + k] = acc;
        }
}

void orc_blank_expansion(const double *Bl, const double *d_old, int H, int S, double *dphi) {
    const int W = S + 1;
    for (int h = 0; h < H; ++h) {
        double acc = 0.0;
        int t2 = S + 1;
        if (g_mutant == 6) t2 = S; /* planted: stop one frame short */
        for (int t1 = 1; t1 <= S; ++t1)
            acc += d_old[(size_t)h * S + (t1 - 1)] * Bl[((size_t)h * W + (t1 - 1)) * W + (t2 - 1)];
        dphi[h] = acc;
    }
}

double orc_round_bf16(double x) {
    float f = (float)x; /* nearest even */
    uint32_t bits;
    memcpy(&bits, &f, 4);
    if ((bits & 0x7F800000u) == 0x7F800000u) return (double)f; /* inf / nan unchanged */
    uint32_t lsb = (bits >> 16) & 1u;
    bits += 0x7FFFu + lsb;
    bits &= 0xFFFF0000u;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/* ================================================================== */
/* LSTM transducer model                                               */
/* ================================================================== */

struct orc_lstm_model {
    orc_lstm_weights w;
    const double *enc;
    int T;
    int n_states, cap;
    size_t stride; /* doubles per state: Dj + 2*layers*H */
    double *store;
};

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

orc_lstm_model *orc_lstm_create(const orc_lstm_weights *w, const double *enc, int T) {
    orc_lstm_model *m = (orc_lstm_model *)calloc(1, sizeof(*m));
    m->w = *w;
    m->enc = enc;
    m->T = T;
    m->stride = (size_t)w->d_joint + 2u * (size_t)w->layers * (size_t)w->hidden;
    m->cap = 64;
    m->store = (double *)malloc(m->stride * (size_t)m->cap * sizeof(double));
    return m;
}

void orc_lstm_destroy(orc_lstm_model *m) {
    if (!m) return;
    free(m->store);
    free(m);
}

static double *state_ptr(orc_lstm_model *m, int s) { return m->store + m->stride * (size_t)s; }

static int new_state(orc_lstm_model *m) {
    if (m->n_states == m->cap) {
        m->cap *= 2;
        m->store = (double *)realloc(m->store, m->stride * (size_t)m->cap * sizeof(double));
    }
    return m->n_states++;
}

int orc_lstm_init_state(orc_lstm_model *m) {
    /* InitPredictor (Section 3.2, helper functions): the predictor output of
     * the empty hypothesis is a given vector; the recurrent state starts at 0. */
    int s = new_state(m);
    double *st = state_ptr(m, s);
    memcpy(st, m->w.pred_init, sizeof(double) * (size_t)m->w.d_joint);
    memset(st + m->w.d_joint, 0, sizeof(double) * 2u * (size_t)m->w.layers * (size_t)m->w.hidden);
    return s;
}

int orc_lstm_update_state(orc_lstm_model *m, int parent_state, int token) {
    /* UpdatePredictorOutput for one hypothesis (Algorithm 1; Section 3.1,
     * g(u) = predictor(y)): embedding, LSTM layers, projection to Dj. */
    const orc_lstm_weights *w = &m->w;
    const int H = w->hidden, L = w->layers, Dj = w->d_joint;
    int s = new_state(m);
    double *st = state_ptr(m, s);
    const double *pa = state_ptr(m, parent_state);
    const double *h_par = pa + Dj;
    const double *c_par = pa + Dj + (size_t)L * H;
    double *h_new = st + Dj;
    double *c_new = st + Dj + (size_t)L * H;
    double *gates = (double *)malloc(sizeof(double) * 4u * (size_t)H);
    double *xin = (double *)malloc(sizeof(double) * (size_t)(w->embed_dim > H ? w->embed_dim : H));
    double *hin = (double *)malloc(sizeof(double) * (size_t)H);
    int in_dim = w->embed_dim;
    for (int i = 0; i < in_dim; ++i) xin[i] = w->embed[(size_t)token * w->embed_dim + i];
    for (int l = 0; l < L; ++l) {
        for (int i = 0; i < H; ++i) {
            double v = h_par[(size_t)l * H + i];
            hin[i] = w->quant_bf16 ? orc_round_bf16(v) : v;
        }
        for (int g = 0; g < 4 * H; ++g) {
            double acc = w->b[l][g];
            const double *wi = w->w_ih[l] + (size_t)g * in_dim;
            for (int i = 0; i < in_dim; ++i) acc += wi[i] * xin[i];
            const double *wh = w->w_hh[l] + (size_t)g * H;
            for (int i = 0; i < H; ++i) acc += wh[i] * hin[i];
            gates[g] = acc;
        }
        for (int i = 0; i < H; ++i) {
            double ig = sigmoid(gates[i]);
            double fg = sigmoid(gates[H + i]);
            double gg = tanh(gates[2 * H + i]);
            double og = sigmoid(gates[3 * H + i]);
            double c = fg * c_par[(size_t)l * H + i] + ig * gg;
            c_new[(size_t)l * H + i] = c;
            h_new[(size_t)l * H + i] = og * tanh(c);
        }
        in_dim = H;
        for (int i = 0; i < H; ++i) {
            double v = h_new[(size_t)l * H + i];
            xin[i] = w->quant_bf16 ? orc_round_bf16(v) : v;
        }
    }
    /* xin now holds the (possibly rounded) top-layer output */
    for (int j = 0; j < Dj; ++j) {
        double acc = w->b_proj[j];
        const double *wp = w->w_proj + (size_t)j * H;
        for (int i = 0; i < H; ++i) acc += wp[i] * xin[i];
        st[j] = acc;
    }
    free(gates);
    free(xin);
    free(hin);
    return s;
}

void orc_lstm_joiner_vec(const orc_lstm_weights *w, const double *e, const double *p, double *logits) {
    /* Joiner (Section 3.1, j(t,u,k) = joiner(h,g)); form: an activation of the
     * sum of the two projected inputs followed by one dense layer
     * (Section 4.1 describes a single activation layer plus one dense layer). */
    const int Dj = w->d_joint, V = w->vocab;
    double *a = (double *)malloc(sizeof(double) * (size_t)Dj);
    for (int j = 0; j < Dj; ++j) {
        double x = e[j] + p[j];
        double v = w->act == 0 ? tanh(x) : (x > 0.0 ? x : 0.0);
        a[j] = w->quant_bf16 ? orc_round_bf16(v) : v;
    }
    for (int k = 0; k < V; ++k) {
        double acc = w->b_out[k];
        const double *wk = w->w_out + (size_t)k * Dj;
        for (int j = 0; j < Dj; ++j) acc += wk[j] * a[j];
        logits[k] = acc;
    }
    free(a);
}

void orc_lstm_joiner(orc_lstm_model *m, int frame, int state, double *logits) {
    orc_lstm_joiner_vec(&m->w, m->enc + (size_t)frame * m->w.d_joint, state_ptr(m, state), logits);
}

void orc_lstm_get_state(const orc_lstm_model *m, int state, double *p, double *h, double *c) {
    const double *st = m->store + m->stride * (size_t)state;
    const size_t LH = (size_t)m->w.layers * m->w.hidden;
    if (p) memcpy(p, st, sizeof(double) * (size_t)m->w.d_joint);
    if (h) memcpy(h, st + m->w.d_joint, sizeof(double) * LH);
    if (c) memcpy(c, st + m->w.d_joint + LH, sizeof(double) * LH);
}

static int lstm_init_cb(void *u) { return orc_lstm_init_state((orc_lstm_model *)u); }
static int lstm_update_cb(void *u, int ps, int tok) { return orc_lstm_update_state((orc_lstm_model *)u, ps, tok); }
static void lstm_joiner_cb(void *u, int f, int s, double *l) { orc_lstm_joiner((orc_lstm_model *)u, f, s, l); }

void orc_lstm_as_model(orc_lstm_model *m, orc_model *out) {
    out->user = m;
    out->vocab = m->w.vocab;
    out->blank_id = m->w.blank_id;
    out->init_state = lstm_init_cb;
    out->update_state = lstm_update_cb;
    out->joiner = lstm_joiner_cb;
}

/* ================================================================== */
/* Hypothesis lists                                                    */
/* ================================================================== */

typedef struct {
    int *tok;
    int len;
    double s;    /* log score (default) or raw probability (raw_prob) */
    int state;   /* predictor state id, -1 = Null */
    double *d;   /* last-token frame distribution, NULL = Null */
    long order;  /* insertion order, for ties */
} hyp;

typedef struct {
    hyp *v;
    int n, cap;
} hlist;

static void hl_init(hlist *l) { l->v = NULL; l->n = 0; l->cap = 0; }

static void hyp_release(hyp *h) {
    free(h->tok);
    free(h->d);
    h->tok = NULL;
    h->d = NULL;
}

static void hl_clear(hlist *l) {
    for (int i = 0; i < l->n; ++i) hyp_release(&l->v[i]);
    l->n = 0;
}

static void hl_free(hlist *l) {
    hl_clear(l);
    free(l->v);
    l->v = NULL;
    l->cap = 0;
}

static hyp *hl_push(hlist *l) {
    if (l->n == l->cap) {
        l->cap = l->cap ? 2 * l->cap : 16;
        l->v = (hyp *)realloc(l->v, sizeof(hyp) * (size_t)l->cap);
    }
    hyp *h = &l->v[l->n++];
    memset(h, 0, sizeof(*h));
    h->state = -1;
    return h;
}

static int *tok_copy(const int *tok, int len, int extra) {
    int *t = (int *)malloc(sizeof(int) * (size_t)(len + extra + 1));
    if (len) memcpy(t, tok, sizeof(int) * (size_t)len);
    return t;
}

static int same_tokens(const hyp *a, const int *tok, int len) {
    if (a->len != len) return 0;
    for (int i = 0; i < len; ++i)
        if (a->tok[i] != tok[i]) return 0;
    return 1;
}

/* ================================================================== */
/* Result and trace                                                    */
/* ================================================================== */

struct orc_result {
    int n;
    int *lens;
    int **tok;
    double *logs;
    long joiner_calls, joined_frames, frames;
    double min_gap;   /* smallest gap of any decision of the run */
    double final_gap; /* gap of the last ChooseNBest(B) alone */
    int *it;
    long n_it, cap_it;
    double *dt;
    long n_dt, cap_dt;
};

static void tr_i(orc_result *r, int v) {
    if (r->n_it == r->cap_it) {
        r->cap_it = r->cap_it ? 2 * r->cap_it : 1024;
        r->it = (int *)realloc(r->it, sizeof(int) * (size_t)r->cap_it);
    }
    r->it[r->n_it++] = v;
}

static void tr_d(orc_result *r, double v) {
    if (r->n_dt == r->cap_dt) {
        r->cap_dt = r->cap_dt ? 2 * r->cap_dt : 1024;
        r->dt = (double *)realloc(r->dt, sizeof(double) * (size_t)r->cap_dt);
    }
    r->dt[r->n_dt++] = v;
}

static void tr_tokens(orc_result *r, const hyp *h) {
    tr_i(r, h->len);
    for (int i = 0; i < h->len; ++i) tr_i(r, h->tok[i]);
}

/* ================================================================== */
/* Helper functions of Algorithm 1                                     */
/* ================================================================== */

typedef struct {
    double key;
    long order;
    int idx;
} rank_item;

static int rank_cmp(const void *a, const void *b) {
    const rank_item *x = (const rank_item *)a, *y = (const rank_item *)b;
    if (x->key > y->key) return -1;
    if (x->key < y->key) return 1;
    if (x->order < y->order) return -1;
    if (x->order > y->order) return 1;
    return 0;
}

/* distance between two scores as |log a - log b| */
static double score_gap(double a, double b, int raw) {
    if (raw) {
        if (a <= 0.0 || b <= 0.0) return INFINITY;
        return fabs(log(a) - log(b));
    }
    if (isinf(a) || isinf(b)) return INFINITY;
    return fabs(a - b);
}

/* A ranking that keeps the best N of n sorted entries decides one thing that
 * rounding could change: which of the N-th and the (N+1)-th entry stays.  The
 * distance between those two is the gap of the decision (infinite when
 * nothing is cut).  The order inside the kept N changes no later score. */
static double cut_gap(const rank_item *sorted, int n, int N, int raw) {
    if (n <= N || N < 1) return INFINITY;
    return score_gap(sorted[N - 1].key, sorted[N].key, raw);
}

static void note_gap(orc_result *r, double g) {
    if (r && g < r->min_gap) r->min_gap = g;
}

/* ChooseNBest: the N highest-scoring hypotheses of src, moved into dst in
 * descending order; the rest are released.  Returns the gap of the cut. */
static double choose_n_best(hlist *src, int N, hlist *dst, orc_result *r, int raw) {
    int n = src->n;
    rank_item *it = (rank_item *)malloc(sizeof(rank_item) * (size_t)(n > 0 ? n : 1));
    for (int i = 0; i < n; ++i) {
        it[i].key = src->v[i].s;
        it[i].order = src->v[i].order;
        it[i].idx = i;
    }
    qsort(it, (size_t)n, sizeof(rank_item), rank_cmp);
    const double gap = cut_gap(it, n, N, raw);
    note_gap(r, gap);
    for (int i = 0; i < n; ++i) {
        hyp *h = &src->v[it[i].idx];
        if (i < N) {
            hyp *o = hl_push(dst);
            *o = *h;
            o->order = i;
            h->tok = NULL;
            h->d = NULL;
        } else {
            hyp_release(h);
        }
    }
    src->n = 0;
    free(it);
    return gap;
}

/* AddAndMerge: append, or add the score to an entry with the same tokens. */
static void add_and_merge(hlist *B, const int *tok, int len, double s, int state, int raw, long *order_ctr) {
    if (g_mutant != 8) {
        for (int i = 0; i < B->n; ++i) {
            if (same_tokens(&B->v[i], tok, len)) {
                double a = B->v[i].s;
                if (g_mutant == 4) { /* planted: keep the larger instead of the sum */
                    B->v[i].s = a > s ? a : s;
                    return;
                }
                if (raw) {
                    B->v[i].s = a + s;
                } else {
                    double mx = a > s ? a : s, mn = a > s ? s : a;
                    B->v[i].s = isinf(mx) ? mx : mx + log1p(exp(mn - mx));
                }
                return;
            }
        }
    }
    hyp *h = hl_push(B);
    h->tok = tok_copy(tok, len, 0);
    h->len = len;
    h->s = s;
    h->state = state;
    h->d = NULL;
    h->order = (*order_ctr)++;
}

/* ChooseNthScore: the N-th highest score of a list with at least N entries. */
static double choose_nth_score(const hlist *B, int N) {
    int n = B->n;
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    for (int i = 0; i < n; ++i) s[i] = B->v[i].s;
    /* selection by repeated maximum: plain and small */
    if (g_mutant == 11 && N < n) N = N + 1; /* planted: one place too far down the list */
    double nth = 0.0;
    for (int r = 0; r < N; ++r) {
        int best = -1;
        for (int i = 0; i < n; ++i)
            if (!isnan(s[i]) && (best < 0 || s[i] > s[best])) best = i;
        nth = s[best];
        s[best] = NAN;
    }
    free(s);
    return nth;
}

/* ================================================================== */
/* Algorithm 1                                                         */
/* ================================================================== */

/* Scores of one round of the inner loop for the H hypotheses of A over the
 * S' frames of the segment that starts at frame t0: the joiner on every
 * (hypothesis, frame) pair, softmax, then Eq. 3-7 in the order of the paper. */
typedef struct {
    int H, Sp, V;
    double *d_old; /* [H][S']     frame distributions the hypotheses came with */
    double *d;     /* [H][V][S']  Eq. 4-5 */
    double *dnb;   /* [H][V]      Eq. 6 */
    double *dphi;  /* [H]         Eq. 7 */
} round_scores;

static void round_scores_free(round_scores *rs) {
    free(rs->d_old);
    free(rs->d);
    free(rs->dnb);
    free(rs->dphi);
}

static round_scores score_round(const orc_model *m, const hlist *A, int t0, int Sp) {
    const int H = A->n, V = m->vocab, blank = m->blank_id;
    round_scores rs;
    rs.H = H;
    rs.Sp = Sp;
    rs.V = V;
    double *logits = (double *)malloc(sizeof(double) * (size_t)H * Sp * V);
    double *J = (double *)malloc(sizeof(double) * (size_t)H * Sp * V);
    double *Bl = (double *)malloc(sizeof(double) * (size_t)H * (Sp + 1) * (Sp + 1));
    rs.d_old = (double *)malloc(sizeof(double) * (size_t)H * Sp);
    rs.d = (double *)malloc(sizeof(double) * (size_t)H * V * Sp);
    rs.dnb = (double *)malloc(sizeof(double) * (size_t)H * V);
    rs.dphi = (double *)malloc(sizeof(double) * (size_t)H);

    /* the joiner sees every frame of the segment with every hypothesis' predictor output
     * (Algorithm 1, first statement of the inner loop; Section 3.1) */
    for (int h = 0; h < H; ++h)
        for (int tau = 0; tau < Sp; ++tau)
            m->joiner(m->user, t0 + tau, A->v[h].state, logits + ((size_t)h * Sp + tau) * V);
    orc_softmax(logits, H * Sp, V, J);

    for (int h = 0; h < H; ++h)
        for (int tau = 0; tau < Sp; ++tau) rs.d_old[(size_t)h * Sp + tau] = A->v[h].d[tau];
    if (g_mutant == 5) /* planted: forget where the last token was emitted */
        for (int h = 0; h < H; ++h) {
            double tot = 0.0;
            for (int tau = 0; tau < Sp; ++tau) tot += rs.d_old[(size_t)h * Sp + tau];
            for (int tau = 0; tau < Sp; ++tau) rs.d_old[(size_t)h * Sp + tau] = tau == 0 ? tot : 0.0;
        }
    orc_blank_product(J, H, Sp, V, blank, Bl);                         /* Eq. 3 */
    orc_nonblank_expansion_t(J, Bl, rs.d_old, H, Sp, V, blank, rs.d);  /* Eq. 4-5 */
    orc_nonblank_expansion(rs.d, H, Sp, V, rs.dnb);                    /* Eq. 6 */
    orc_blank_expansion(Bl, rs.d_old, H, Sp, rs.dphi);                 /* Eq. 7 */
    free(logits);
    free(J);
    free(Bl);
    return rs;
}

/* Every hypothesis of A may stop emitting in this segment: its blank expansion
 * (Eq. 7) goes into B, merged with an entry of equal tokens if there is one
 * (Algorithm 1, the loop over AddAndMerge). */
static void merge_blank_expansions(hlist *B, const hlist *A, const round_scores *rs, int raw, long *order_ctr) {
    for (int h = 0; h < A->n; ++h) {
        double sc = raw ? rs->dphi[h] : A->v[h].s + log(rs->dphi[h]);
        add_and_merge(B, A->v[h].tok, A->v[h].len, sc, A->v[h].state, raw, order_ctr);
    }
}

/* The next A: of all (hypothesis, non-blank token) pairs the N with the best
 * non-blank expansion score (Eq. 6) are looked at, best first, and one becomes
 * a hypothesis if B is still short of N entries or its score beats the N-th
 * score of B (Algorithm 1: ChooseNthScore, ChooseNBestExpansions and the test
 * inside the loop over them).  A new hypothesis takes the tokens of its parent
 * plus the token, the expansion score, no predictor output yet, and the frame
 * distribution of that token (Eq. 5).  new_pairs receives (parent, token) of
 * each; *threshold_out the threshold (NaN when B is short); the return value
 * is the smallest gap of the decisions taken here. */
static double select_expansions(const hlist *A, const hlist *B, const round_scores *rs, int N, int blank, int raw,
                                hlist *An, int *new_pairs, double *threshold_out) {
    const int H = rs->H, V = rs->V, Sp = rs->Sp;
    double gap = INFINITY;
    const int have_thr = B->n >= N;
    const double threshold = have_thr ? choose_nth_score(B, N) : NAN;
    *threshold_out = threshold;

    size_t ncand = 0;
    rank_item *cand = (rank_item *)malloc(sizeof(rank_item) * (size_t)H * V);
    for (int h = 0; h < H; ++h)
        for (int k = 0; k < V; ++k) {
            if (k == blank) continue;
            double p = rs->dnb[(size_t)h * V + k];
            if (!(p > 0.0)) continue;
            cand[ncand].key = raw ? p : A->v[h].s + log(p);
            cand[ncand].order = (long)h * V + k;
            cand[ncand].idx = h * V + k;
            ++ncand;
        }
    qsort(cand, ncand, sizeof(rank_item), rank_cmp);
    int ntop = (int)ncand < N ? (int)ncand : N;
    if (g_mutant == 10) { /* planted: the N best of every hypothesis instead of the N best of all */
        size_t w = 0;
        int *taken = (int *)calloc((size_t)H, sizeof(int));
        for (size_t i = 0; i < ncand; ++i)
            if (taken[cand[i].idx / V]++ < N) cand[w++] = cand[i];
        free(taken);
        ntop = (int)w;
    } else if (ntop == N && (!have_thr || cand[N - 1].key > threshold)) {
        /* the cut after the N-th pair matters only if that pair is kept */
        double g = cut_gap(cand, (int)ncand, N, raw);
        if (g < gap) gap = g;
    }

    hl_clear(An);
    for (int i = 0; i < ntop; ++i) {
        int h = cand[i].idx / V, k = cand[i].idx % V;
        double key = cand[i].key;
        if (have_thr) {
            double g = score_gap(key, threshold, raw);
            if (g < gap) gap = g;
        }
        int keep = (B->n < N) || (g_mutant == 9 ? key >= threshold /* planted: not strict */ : key > threshold);
        if (!keep) continue;
        hyp *nh = hl_push(An);
        nh->tok = tok_copy(A->v[h].tok, A->v[h].len, 1);
        nh->tok[A->v[h].len] = k;
        nh->len = A->v[h].len + 1;
        nh->s = key;
        nh->state = A->v[h].state; /* the parent's, until the predictor has run */
        nh->d = (double *)malloc(sizeof(double) * (size_t)Sp);
        double norm = raw ? 1.0 : rs->dnb[(size_t)h * V + k];
        for (int tau = 0; tau < Sp; ++tau) nh->d[tau] = rs->d[((size_t)h * V + k) * Sp + tau] / norm;
        nh->order = An->n - 1;
        new_pairs[2 * (An->n - 1)] = h;
        new_pairs[2 * (An->n - 1) + 1] = k;
    }
    free(cand);
    return gap;
}

/*
 * Trace layout (opts.trace = 1).  One record per round of the inner loop.
 *  int stream:    -1, segment, round, S', H, nB, nA_new,
 *                 then for each incoming hypothesis h: len, tokens...
 *                 then for each entry of B after the merges: len, tokens...
 *                 then for each new hypothesis: parent h, token k
 *  double stream: for each incoming h: score in, delta_blank (relative to the score
 *                   unless raw_prob), then the S' entries of d_old
 *                 threshold (NaN when B holds fewer than N)
 *                 scores of B after the merges (nB)
 *                 for each new hypothesis: score, then the S' entries of its d
 *                 gap of the ChooseNBest that opened this segment, smallest gap of this round's decisions
 */
orc_result *orc_decode(const orc_model *m, int T, const orc_search_opts *o) {
    const int N = o->beam_n, S = o->seg_s, blank = m->blank_id, raw = o->raw_prob;
    orc_result *res = (orc_result *)calloc(1, sizeof(*res));
    res->min_gap = INFINITY;
    res->final_gap = INFINITY;
    res->frames = T;

    hlist A, B, An;
    hl_init(&A);
    hl_init(&B);
    hl_init(&An);
    long order_ctr = 0;

    /* B starts as the empty hypothesis with score one and the initial predictor output */
    {
        hyp *h = hl_push(&B);
        h->tok = tok_copy(NULL, 0, 0);
        h->len = 0;
        h->s = raw ? 1.0 : 0.0;
        h->state = m->init_state(m->user);
        h->order = order_ctr++;
    }

    int t = 0, seg_index = 0;
    while (t < T) {
        /* head of the outer loop: the next S frames (fewer at the end), A = the N best of B,
         * B emptied, every d set to (score, 0, ..., 0) */
        const int Sp = (T - t) < S ? (T - t) : S;
        hl_clear(&A);
        const double head_gap = choose_n_best(&B, N, &A, res, raw);
        order_ctr = 0;
        for (int h = 0; h < A.n; ++h) {
            free(A.v[h].d);
            A.v[h].d = (double *)calloc((size_t)Sp, sizeof(double));
            A.v[h].d[0] = raw ? A.v[h].s : 1.0;
        }
        int round = 0;
        while (A.n > 0) {
            ++round;
            const int H = A.n;
            round_scores rs = score_round(m, &A, t, Sp);
            res->joiner_calls += 1;
            res->joined_frames += Sp;

            if (o->trace) {
                tr_i(res, -1); tr_i(res, seg_index); tr_i(res, round); tr_i(res, Sp); tr_i(res, H);
            }
            const long trace_counts_at = res->n_it;
            if (o->trace) {
                tr_i(res, 0); tr_i(res, 0); /* nB and nA_new, filled in below */
                for (int h = 0; h < H; ++h) tr_tokens(res, &A.v[h]);
                for (int h = 0; h < H; ++h) {
                    tr_d(res, A.v[h].s);
                    tr_d(res, rs.dphi[h]);
                    for (int tau = 0; tau < Sp; ++tau) tr_d(res, rs.d_old[(size_t)h * Sp + tau]);
                }
            }

            merge_blank_expansions(&B, &A, &rs, raw, &order_ctr);
            int *new_pairs = (int *)malloc(sizeof(int) * (size_t)(2 * (size_t)H * N + 2));
            double threshold;
            const double round_gap = select_expansions(&A, &B, &rs, N, blank, raw, &An, new_pairs, &threshold);
            note_gap(res, round_gap);

            if (o->trace) {
                res->it[trace_counts_at] = B.n;
                res->it[trace_counts_at + 1] = An.n;
                for (int i = 0; i < B.n; ++i) tr_tokens(res, &B.v[i]);
                for (int i = 0; i < 2 * An.n; ++i) tr_i(res, new_pairs[i]);
                tr_d(res, threshold);
                for (int i = 0; i < B.n; ++i) tr_d(res, B.v[i].s);
                for (int i = 0; i < An.n; ++i) {
                    tr_d(res, An.v[i].s);
                    for (int tau = 0; tau < Sp; ++tau) tr_d(res, An.v[i].d[tau]);
                }
                tr_d(res, head_gap);
                tr_d(res, round_gap);
            }
            free(new_pairs);
            round_scores_free(&rs);

            /* the predictor runs once for every new hypothesis (UpdatePredictorOutput) */
            for (int i = 0; i < An.n; ++i)
                An.v[i].state = m->update_state(m->user, An.v[i].state, An.v[i].tok[An.v[i].len - 1]);

            /* the new hypotheses are the A of the next round */
            hl_clear(&A);
            hlist tmp = A;
            A = An;
            An = tmp;

            if (o->max_rounds > 0 && round >= o->max_rounds) hl_clear(&A);
        }
        t += S;
        ++seg_index;
    }

    /* the result is the N best of B */
    hlist out;
    hl_init(&out);
    res->final_gap = choose_n_best(&B, N, &out, res, raw);
    res->n = out.n;
    res->lens = (int *)malloc(sizeof(int) * (size_t)(out.n + 1));
    res->tok = (int **)malloc(sizeof(int *) * (size_t)(out.n + 1));
    res->logs = (double *)malloc(sizeof(double) * (size_t)(out.n + 1));
    for (int i = 0; i < out.n; ++i) {
        res->lens[i] = out.v[i].len;
        res->tok[i] = out.v[i].tok;
        out.v[i].tok = NULL;
        res->logs[i] = raw ? log(out.v[i].s) : out.v[i].s;
    }
    hl_free(&out);
    hl_free(&A);
    hl_free(&An);
    hl_free(&B);
    return res;
}

void orc_result_free(orc_result *r) {
    if (!r) return;
    for (int i = 0; i < r->n; ++i) free(r->tok[i]);
    free(r->tok);
    free(r->lens);
    free(r->logs);
    free(r->it);
    free(r->dt);
    free(r);
}

int orc_result_count(const orc_result *r) { return r->n; }
int orc_result_len(const orc_result *r, int i) { return r->lens[i]; }
const int *orc_result_tokens(const orc_result *r, int i) { return r->tok[i]; }
double orc_result_logscore(const orc_result *r, int i) { return r->logs[i]; }

void orc_result_counters(const orc_result *r, long *joiner_calls, long *joined_frames, long *frames) {
    if (joiner_calls) *joiner_calls = r->joiner_calls;
    if (joined_frames) *joined_frames = r->joined_frames;
    if (frames) *frames = r->frames;
}

double orc_result_min_gap(const orc_result *r) { return r->min_gap; }
double orc_result_final_gap(const orc_result *r) { return r->final_gap; }

long orc_result_trace(const orc_result *r, const int **itrace, long *n_i, const double **dtrace, long *n_d) {
    *itrace = r->it;
    *n_i = r->n_it;
    *dtrace = r->dt;
    *n_d = r->n_dt;
    return r->n_it;
}

int orc_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int orc_decode_lstm_batch(const orc_lstm_weights *w, const double *enc, const int *offsets, int U,
                          const orc_search_opts *o, int threads, orc_result **res) {
    int used = 1;
#ifdef _OPENMP
    if (threads < 1) threads = 1;
    used = threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
    for (int u = 0; u < U; ++u) {
        int T = offsets[u + 1] - offsets[u];
        orc_lstm_model *m = orc_lstm_create(w, enc + (size_t)offsets[u] * w->d_joint, T);
        orc_model mm;
        orc_lstm_as_model(m, &mm);
        res[u] = orc_decode(&mm, T, o);
        orc_lstm_destroy(m);
    }
    return used;
}
