/*
 * CPU oracle for token-wise RNN-T beam search (Keren, "A Token-Wise Beam
 * Search Algorithm for RNN-T", Algorithm 1 and Eq. 1-7).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 implementation that
 * follows the paper step by step and shares no code with the HIP library.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  The product path never does.
 *
 * Score domain.  The paper keeps raw probabilities starting from score 1.
 * Over hundreds of frames these underflow, so by default a hypothesis keeps
 * log(score) and a frame distribution d normalised to sum to one; Eq. 3-7 are
 * linear in d_old, so working on d/score and adding log(score) back is the
 * same arithmetic.  With raw_prob=1 the driver keeps raw probabilities exactly
 * as printed (short inputs only); tests check the two agree.
 *
 * Pins (tests/, CPU): brute-force enumeration of every alignment on tiny
 * lattices, conservation of probability mass through Eq. 3-7, S=1 against an
 * independently written frame-wise search (Eq. 1), the transducer forward
 * recursion with pruning disabled for every S, and library routines for
 * softmax / LSTM cell / dense layers / bf16 rounding.  The beam policy itself
 * (threshold rule, strict '>', joint top-N, tie order) is fixed only by the
 * text of Algorithm 1: parity unpinned beyond that reading.
 */
#ifndef TBS_ORACLE_H
#define TBS_ORACLE_H

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------ */
/* Score algebra of one joiner call: H hypotheses, S frames, V symbols */
/* ------------------------------------------------------------------ */

/* Softmax over each row of V logits (Algorithm 1, the line that forms J;
 * Section 3.1: J is the joiner output after softmax normalisation). */
void orc_softmax(const double *logits, int rows, int V, double *J);

/* Eq. 3.  J is [H][S][V].  Bl is [H][S+1][S+1]; entry [h][t1-1][t2-1] holds
 * Bl(h, t1, t2) for 1 <= t1, t2 <= S+1: the product of blank probabilities of
 * frames t1 .. t2-1, one when t1 == t2, zero when t1 > t2. */
void orc_blank_product(const double *J, int H, int S, int V, int blank, double *Bl);

/* Eq. 4 and 5.  d_old is [H][S]; d is [H][V][S] with
 * d[h][k][t2] = sum_{t1} d_old[h][t1] * Bl(h,t1,t2) * J[h][t2][k]; the blank
 * column of d is set to zero (blank is not a non-blank expansion). */
void orc_nonblank_expansion_t(const double *J, const double *Bl, const double *d_old,
                              int H, int S, int V, int blank, double *d);

/* Eq. 6.  dnb [H][V] = sum over t2 of d. */
void orc_nonblank_expansion(const double *d, int H, int S, int V, double *dnb);

/* Eq. 7.  dphi [H] = sum_{t1} d_old[h][t1] * Bl(h, t1, S+1). */
void orc_blank_expansion(const double *Bl, const double *d_old, int H, int S, double *dphi);

/* Round a value to bf16 precision the way a kernel holding it in fp32 does:
 * to float (nearest even), then to the upper 16 bits (nearest even). */
double orc_round_bf16(double x);

/* Tests only: a value other than zero plants one known mistake in the code
 * above or in the driver, to show that the pins notice it.  0 restores. */
void orc_set_mutant(int m);

/* ------------------------------------------------------------------ */
/* Model interface used by the search driver                           */
/* ------------------------------------------------------------------ */

typedef struct orc_model {
    void *user;
    int vocab;     /* V, including blank */
    int blank_id;
    /* InitPredictor(): state id of the empty hypothesis */
    int (*init_state)(void *user);
    /* UpdatePredictorOutput for one hypothesis: state after appending token */
    int (*update_state)(void *user, int parent_state, int token);
    /* Joiner for one (frame, hypothesis) pair: V logits, before softmax.
     * frame is the 0-based index into the utterance. */
    void (*joiner)(void *user, int frame, int state, double *logits);
} orc_model;

/* ------------------------------------------------------------------ */
/* LSTM transducer model (embedding + LSTM layers + projections)       */
/* ------------------------------------------------------------------ */

typedef struct orc_lstm_weights {
    int d_joint, vocab, blank_id;
    int embed_dim, hidden, layers;
    int act;         /* 0 = tanh, 1 = relu */
    int quant_bf16;  /* 1: round act(e+p) and every h used as a matrix input to bf16 */
    const double *w_out;   /* [V][Dj] */
    const double *b_out;   /* [V] */
    const double *embed;   /* [V][E] */
    const double *w_ih[8]; /* [4H][in_l], gate order i,f,g,o */
    const double *w_hh[8]; /* [4H][H] */
    const double *b[8];    /* [4H] */
    const double *w_proj;  /* [Dj][H] */
    const double *b_proj;  /* [Dj] */
    const double *pred_init; /* [Dj] */
} orc_lstm_weights;

typedef struct orc_lstm_model orc_lstm_model;

/* enc is [T][Dj] projected encoder frames of one utterance (borrowed). */
orc_lstm_model *orc_lstm_create(const orc_lstm_weights *w, const double *enc, int T);
void orc_lstm_destroy(orc_lstm_model *m);
void orc_lstm_as_model(orc_lstm_model *m, orc_model *out);
int orc_lstm_init_state(orc_lstm_model *m);
int orc_lstm_update_state(orc_lstm_model *m, int parent_state, int token);
void orc_lstm_joiner(orc_lstm_model *m, int frame, int state, double *logits);
/* read back a state: p [Dj], h [layers][H], c [layers][H]; any pointer may be NULL */
void orc_lstm_get_state(const orc_lstm_model *m, int state, double *p, double *h, double *c);
/* joiner on explicit vectors: logits = W_out * act(e + p) + b_out */
void orc_lstm_joiner_vec(const orc_lstm_weights *w, const double *e, const double *p, double *logits);

/* ------------------------------------------------------------------ */
/* Search driver (Algorithm 1)                                         */
/* ------------------------------------------------------------------ */

typedef struct orc_search_opts {
    int beam_n;      /* N */
    int seg_s;       /* S */
    int max_rounds;  /* 0: no limit (the paper); >0: drop A after that many rounds per segment */
    int raw_prob;    /* 1: keep raw probabilities as printed; 0: log score + normalised d */
    int trace;       /* 1: record every round (see orc_result_trace) */
} orc_search_opts;

typedef struct orc_result orc_result;

orc_result *orc_decode(const orc_model *m, int T, const orc_search_opts *o);
void orc_result_free(orc_result *r);
int orc_result_count(const orc_result *r);
int orc_result_len(const orc_result *r, int i);
const int *orc_result_tokens(const orc_result *r, int i);
double orc_result_logscore(const orc_result *r, int i);
/* counters: joiner calls, frames joined (summed over calls: rows / hypotheses), frames decoded */
void orc_result_counters(const orc_result *r, long *joiner_calls, long *joined_frames, long *frames);
/* Smallest |log a - log b| over the decisions of the run that rounding could turn: the N-th
 * against the (N+1)-th entry wherever a ranking keeps N (ChooseNBest at the head of a segment
 * and at the end, ChooseNBestExpansions when its N-th pair is kept), and every expansion score
 * against the threshold it is tested with.  A run whose smallest gap exceeds the tolerance of a
 * comparison has one correct output; the trace holds the gap of every segment head and round. */
double orc_result_min_gap(const orc_result *r);
/* the same for the last ChooseNBest(B) alone (infinite if B held at most N entries) */
double orc_result_final_gap(const orc_result *r);
/* trace: flat int and double streams, layout documented in tbs_oracle.c */
long orc_result_trace(const orc_result *r, const int **itrace, long *n_i, const double **dtrace, long *n_d);

/* Decode U utterances with the LSTM model, OpenMP-parallel over utterances.
 * enc [sum T][Dj], offsets [U+1].  Results: res[u] (caller frees each). */
int orc_decode_lstm_batch(const orc_lstm_weights *w, const double *enc, const int *offsets, int U,
                          const orc_search_opts *o, int threads, orc_result **res);
int orc_max_threads(void);

#ifdef __cplusplus
}
#endif
#endif
