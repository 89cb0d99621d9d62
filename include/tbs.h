/*
 * tbs - token-wise beam search for RNN-T on one AMD MI355X (gfx950).
 *
 * C ABI of the hot path of token-wise RNN-T beam search (Keren, "A Token-Wise
 * Beam Search Algorithm for RNN-T"): per decoding segment of S encoder frames,
 * a batched joiner over (frames x live hypotheses x vocabulary), softmax
 * statistics, the blank / non-blank expansion scores of Eq. 3-7, N-best
 * selection with merging of equal token sequences, and the predictor update.
 * Every step runs in HIP kernels; nothing here falls back to the CPU.
 *
 * Conventions
 *  - "DEVICE" pointers are HIP device memory on the context's device; "HOST"
 *    pointers are ordinary host memory.  The caller owns every buffer it
 *    passes; weights and encoder frames are borrowed and must outlive their
 *    use (weights: the context; frames: until the next tbs_begin/tbs_decode).
 *  - All matrices are row-major [out_features, in_features] (the reduction
 *    index is contiguous).  dtype 0: float32 everywhere.  dtype 1: matrices
 *    and encoder frames are bf16, biases and predictor outputs float32,
 *    accumulation float32.
 *  - Scores are natural-log probabilities (float64 in bookkeeping); the frame
 *    distribution d of a hypothesis is stored normalised to sum to one
 *    (Eq. 3-7 are linear in it), so nothing underflows over long utterances.
 *  - Every call returns 0 or a negative TBS_E* code; nothing throws or aborts.
 *    Kernels are enqueued on the context's stream; calls that take a HOST
 *    output pointer synchronise that stream before returning.
 *  - A context is not thread-safe.
 */
#ifndef TBS_H
#define TBS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TBS_OK 0
#define TBS_EINVAL (-1)    /* bad argument or unsupported shape */
#define TBS_ESTATE (-2)    /* call out of order */
#define TBS_ENOMEM (-3)    /* device or host allocation failed */
#define TBS_EHIP (-4)      /* a HIP call failed; see tbs_last_hip_error */
#define TBS_EOVERFLOW (-5) /* a capacity was exceeded (rounds, merged list, trie nodes, max_len) */
#define TBS_ELIMIT (-6)    /* request larger than the fixed scratch of an entry point that does not allocate */

#define TBS_MAX_BEAM 32
#define TBS_MAX_SEG 128
#define TBS_MAX_LAYERS 4

typedef struct tbs_ctx tbs_ctx;

typedef struct tbs_config {
    int32_t d_joint;          /* Dj: width of the joint space */
    int32_t vocab;            /* V: joiner outputs including blank */
    int32_t blank_id;
    int32_t beam_n;           /* N (Algorithm 1 input), 1..TBS_MAX_BEAM */
    int32_t seg_s;            /* S (Algorithm 1 input), 1..TBS_MAX_SEG */
    int32_t max_utts;         /* capacity: utterances decoded together */
    int32_t max_frames_total; /* capacity: sum of utterance lengths */
    int32_t pred_layers;      /* LSTM layers of the prediction network, 1..TBS_MAX_LAYERS */
    int32_t pred_hidden;
    int32_t pred_embed;       /* token embedding width */
    int32_t act;              /* joiner activation: 0 tanh, 1 relu */
    int32_t dtype;            /* 0 float32, 1 bf16 (see above) */
    int32_t max_rounds_per_segment; /* >0: hypotheses still emitting after that many rounds of a
                                       segment are dropped (the N-step style limit the paper tried
                                       and left out, Section 3.2); 0: no such limit, but more than
                                       rounds_capacity rounds is TBS_EOVERFLOW */
    int32_t rounds_capacity;  /* sizes the per-segment workspaces; 0 = 32 */
    int32_t max_nodes;        /* capacity of the token trie; 0 = 4*N*(max_frames_total+max_utts*S) */
    int32_t debug;            /* bit 0: also keep per-row softmax statistics and the full non-blank
                                 expansion scores for tbs_debug_read; bit 1: always use the
                                 generic two-pass expansion kernel; bit 3: keep the LSTM cell update a
                                 kernel of its own also where it would run inside the gate GEMM;
                                 bit 4: always form the joiner input rows in a kernel of their own,
                                 also where the predictor projection's epilogue would; bit 5: always
                                 gather the first LSTM layer's input rows in a kernel of their own,
                                 also where the row list kernel would; bit 6: enqueue the predictor
                                 step only once the host knows how many hypotheses the round
                                 created, also where it could go out ahead of that; bit 7: keep
                                 expansion and select/merge two kernels inside tbs_decode and
                                 tbs_push_segment also where one kernel would run both; bit 8: keep the
                                 row lists (hypotheses and joiner rows compacted over the batch by a
                                 kernel of its own every round) also where a small batch would run with
                                 every hypothesis in a fixed place and no such kernel; bit 9: with
                                 seg_s = 1 (the standard breadth-first search, Eq. 1) store the logits and
                                 expand from them as for longer segments, also where the joiner GEMM
                                 would keep only each row's softmax sums and best tokens (see bit 15); bit 10: form the
                                 joiner input rows of a segment's first round in a kernel of their own,
                                 also where the kernel that starts the segment would; bit 11: one
                                 workgroup per tile of the predictor projection forms the joiner input rows
                                 of all of a pair's frames, also where a small problem would run one
                                 workgroup per tile and frame; bit 12: the joiner GEMM of a small batch spreads
                                 its tiles over the XCDs as the other GEMMs do, also where it would give every
                                 XCD a range of rows of its own; bit 13: the kernel that forms joiner input
                                 rows takes a thread per row, also where it would take a thread per pair; bit 14:
                                 seg_s = 1 without logits: the joiner GEMM merges the partials of a tile's four
                                 16-column pieces itself, also where it would hand them to the round kernel
                                 as they are; bit 15: seg_s = 1 without logits also where the form with
                                 logits would run (beams above 4 with a vocabulary it can hold, where it was
                                 measured faster; tests cover each pair of variants) */
    int32_t stream_buffer_frames; /* per-utterance capacity, in frames, of the buffer tbs_push_segment
                                 collects encoder frames in; 0 = no streaming.  At least seg_s; one
                                 push may bring an utterance up to this many minus seg_s - 1 frames */
    int32_t max_result_len;   /* longest token sequence tbs_decode / tbs_result hand back (sizes the result
                                 buffer at tbs_init); 0 = 256.  A larger max_len there is TBS_EINVAL */
    int32_t joiner_chunk_rows; /* > 0: a joiner call with more rows than this is run in pieces of about that
                                 many rows (whole hypotheses), each piece expanded right behind its GEMM
                                 while its logits are still in the memory-side cache; 0: never split (the
                                 default: splitting measured slower on this part, see tbs_joiner_segment) */
    int32_t device_id;
    void *stream;             /* hipStream_t to enqueue on (0 = the null stream) */
} tbs_config;

typedef struct tbs_weights {          /* DEVICE pointers, borrowed */
    const void *w_out;                /* [V, Dj]   joiner output layer */
    const float *b_out;               /* [V] */
    const void *embed;                /* [V, E] */
    const void *w_ih[TBS_MAX_LAYERS]; /* [4H, in_l] gate order i,f,g,o; in_0 = E, else H */
    const void *w_hh[TBS_MAX_LAYERS]; /* [4H, H] */
    const float *b_lstm[TBS_MAX_LAYERS]; /* [4H] */
    const void *w_proj;               /* [Dj, H]  predictor output -> joint space */
    const float *b_proj;              /* [Dj] */
    const float *pred_init;           /* [Dj] predictor output of the empty hypothesis (InitPredictor) */
} tbs_weights;

/* Create a context: validates the configuration, allocates every workspace
 * once (no later call of the decode or streaming path allocates; the inspection
 * and timing calls below make temporaries of their own), and prepares the
 * predictor weights.  N * rounds capacity (the longest list B) may not exceed 2048.
 * Algorithm 1 inputs N and S are fixed per context. */
int tbs_init(const tbs_config *cfg, const tbs_weights *w, tbs_ctx **out);
void tbs_free(tbs_ctx *ctx);

/* Bind a batch of U utterances: enc_proj DEVICE [sum T_u, Dj] holds the
 * encoder output frames (Algorithm 1 input enc) already projected to the joint
 * space, ragged; frame_offsets HOST [U+1].  Sets B = [([], 1, InitPredictor(),
 * Null)] for every utterance (Algorithm 1, first line). */
int tbs_begin(tbs_ctx *ctx, const void *enc_proj, const int32_t *frame_offsets, int32_t U);

/* Start segment seg_index (frames seg_index*S ..): A = ChooseNBest(B), B = [],
 * d = (s, 0, ..., 0) for every utterance that still has frames (Algorithm 1,
 * head of the outer loop).  rows_host (HOST, may be NULL) receives the number
 * of joiner rows of the first round. */
int tbs_segment_begin(tbs_ctx *ctx, int32_t seg_index, int32_t *rows_host);

/* J = Softmax(Joiner(seg, pred)) for all live (utterance, hypothesis, frame)
 * rows in one batched call (Algorithm 1, first line of the inner loop;
 * Section 3.1).  Logits are written once; softmax is kept as per-row
 * statistics, the probabilities are never stored.  With joiner_chunk_rows set,
 * a call larger than that is run in pieces and the expansion of each piece
 * follows its GEMM at once, inside this call; tbs_expand, which must still be
 * called next, then finds its work done. */
int tbs_joiner_segment(tbs_ctx *ctx);

/* BlankProduct, NonBlankExpansionT, NonBlankExpansion and BlankExpansion
 * (Eq. 3-7) for every live hypothesis, and its N best non-blank expansions. */
int tbs_expand(tbs_ctx *ctx);

/* AddAndMerge of the blank expansions into B, ChooseNthScore, the joint
 * ChooseNBestExpansions with the threshold test, and the new list A with its
 * frame distributions (Algorithm 1, second half of the inner loop).
 * live_host (HOST, may be NULL) receives the total size of the new A lists. */
int tbs_select_merge(tbs_ctx *ctx, int32_t *live_host);

/* UpdatePredictorOutput(A): embedding, LSTM layers and projection for the
 * hypotheses tbs_select_merge just created. */
int tbs_predictor_step(tbs_ctx *ctx);

/* Algorithm 1 for U utterances in lock-step; equals running each alone.
 * Outputs (HOST): tokens [U, N, max_len], lens [U, N], logscores [U, N]
 * (natural log), nbest_count [U]; hypotheses in descending score order.
 * A hypothesis longer than max_len is truncated to its first max_len tokens (lens
 * still holds its true length) and TBS_EOVERFLOW returned; the other outputs are complete.
 * max_len may not exceed the configuration's max_result_len. */
int tbs_decode(tbs_ctx *ctx, const void *enc_proj, const int32_t *frame_offsets, int32_t U,
               int32_t *tokens, int32_t *lens, double *logscores, int32_t *nbest_count,
               int32_t max_len);

/* Streaming (Section 3.2, the remarks after Algorithm 1: the encoder output may arrive segment by
 * segment, and the segment size of the encoder need not be that of the decoder).
 * tbs_stream_begin binds U utterances with no frames yet (B as after tbs_begin).
 * tbs_push_segment appends the frames enc_proj DEVICE [sum n_u, Dj], ragged by frame_offsets
 * HOST [U+1] (n_u >= 0 new frames of utterance u), to the utterances' buffers and runs Algorithm
 * 1's outer loop for every whole segment of S buffered frames of every utterance, utterances
 * advancing independently; flush != 0 also decodes each utterance's remaining frames as one
 * shorter segment (the end of the utterance; later frames start a new segment).  B is the state
 * kept between calls: tbs_result after any push returns ChooseNBest(B) for the frames decoded so
 * far.  Pushing all frames of a batch in any pieces and flushing at the end gives what tbs_decode
 * gives.  On return the frames have been copied: the caller may reuse enc_proj.
 * TBS_EINVAL (nothing changed) if a buffer would overflow or the frames pushed since
 * tbs_stream_begin would exceed max_frames_total. */
int tbs_stream_begin(tbs_ctx *ctx, int32_t U);
int tbs_push_segment(tbs_ctx *ctx, const void *enc_proj, const int32_t *frame_offsets, int32_t flush);

/* ChooseNBest(B) of every utterance, as tbs_decode returns it (for callers
 * that drive the step functions themselves). */
int tbs_result(tbs_ctx *ctx, int32_t *tokens, int32_t *lens, double *logscores,
               int32_t *nbest_count, int32_t max_len);

/* Counters in the paper's sense (Section 4.2): joiner invocations and frames
 * joined, per utterance summed (an utterance counts a call when it had rows in
 * it), and frames decoded; plus the number of batched joiner launches. */
int tbs_stats(const tbs_ctx *ctx, int64_t *joiner_calls, int64_t *joined_frames, int64_t *frames,
              int64_t *launches);

/* Which forms of the kernels the batch begun last runs in (they give the same results; tests and
 * benchmarks use this to say which one they exercised): bit 0 = every hypothesis in a fixed place,
 * four kernels a round; bit 1 = seg_s = 1 without logits (the standard search of Eq. 1 with the
 * row softmax sums and best tokens made in the joiner GEMM).  Negative: an error code. */
int tbs_path(const tbs_ctx *ctx);

/* ---- inspection, for tests ---- */
enum tbs_buffer {
    TBS_BUF_A_COUNT = 0,   /* int32  [U]        hypotheses in A */
    TBS_BUF_A_LOGS = 1,    /* double [U,N]      log scores of A */
    TBS_BUF_A_DHAT = 2,    /* float  [U,N,S]    normalised frame distributions of A */
    TBS_BUF_A_PRED = 3,    /* float  [U,N,Dj]   projected predictor outputs of A */
    TBS_BUF_LOGITS = 4,    /* float  [rows,V]   joiner logits of the current round */
    TBS_BUF_ROW_STATS = 5, /* float  [rows,3]   row max, sum of exp(l-max), blank probability (debug=1) */
    TBS_BUF_DELTA_BLANK = 6, /* float [pairs]   natural logarithm of the blank expansion score (Eq. 7) relative to
                                                the hypothesis score */
    TBS_BUF_DELTA_NB = 7,  /* float  [pairs,V]  non-blank expansion scores, relative (debug=1) */
    TBS_BUF_CAND_SCORE = 8, /* float [pairs,N]  log of the N best relative scores per hypothesis */
    TBS_BUF_CAND_TOKEN = 9, /* int32 [pairs,N]  their tokens (-1 = none) */
    TBS_BUF_PAIR_UTT = 10, /* int32  [pairs]    utterance of each live hypothesis, in row order */
    TBS_BUF_PAIR_HYP = 11, /* int32  [pairs]    its index in A */
    TBS_BUF_PAIR_ROW0 = 12,/* int32  [pairs]    its first joiner row */
    TBS_BUF_PAIR_LEN = 13, /* int32  [pairs]    its frames in this segment */
    TBS_BUF_COUNTS = 14    /* int32  [4]        pairs, rows, trie nodes used, error flags */
};
/* Copy a buffer to HOST memory (at most `bytes`).  "rows" and "pairs" are the
 * current round's counts (TBS_BUF_COUNTS). */
int tbs_debug_read(tbs_ctx *ctx, int32_t which, void *dst, size_t bytes);
/* Overwrite A_COUNT / A_LOGS / A_DHAT / A_PRED from HOST memory (full arrays),
 * so that a test can put the joiner and expansion steps on chosen inputs.  Not
 * between tbs_select_merge and tbs_predictor_step: part of the predictor step
 * may already have run on the state as it was. */
int tbs_debug_write(tbs_ctx *ctx, int32_t which, const void *src, size_t bytes);
/* After tbs_debug_write: rebuild the row list for segment seg_index without
 * touching A or B. */
int tbs_debug_rebuild(tbs_ctx *ctx, int32_t seg_index, int32_t *rows_host);
/* Token sequences and scores of group A (0) or B (1): tokens [U,cap,max_len],
 * lens [U,cap], logscores [U,cap], counts [U], all HOST. */
int tbs_debug_hyps(tbs_ctx *ctx, int32_t group, int32_t *tokens, int32_t *lens, double *logscores,
                   int32_t *counts, int32_t cap, int32_t max_len);

/* tbs_debug_hyps for callers that cannot allocate device memory (a tight serving loop reading the
 * running hypotheses after every push, a harness that forbids allocation, code that must not
 * call the allocator between captures): the same outputs, but the kernel's staging area is a
 * fixed 2 MiB array in the library's device image instead of four allocations per call, and the
 * call makes no allocation of any kind.  U * cap * (max_len + 3) * 4 + U * 4 bytes (U = utterances
 * of the current batch) must fit into it, otherwise TBS_ELIMIT and nothing is done.  Every GPU
 * holds its own copy of the array from the moment the library is loaded until the process ends;
 * all contexts on one GPU share it, so calls that overlap in time on one GPU (from different
 * contexts or streams) race and must be serialised by the caller.  The array keeps what the last
 * call left in it; the kernel overwrites every entry it hands back. */
int tbs_debug_hyps_noalloc(tbs_ctx *ctx, int32_t group, int32_t *tokens, int32_t *lens, double *logscores,
                           int32_t *counts, int32_t cap, int32_t max_len);

/* ---- timing of one kernel family, for the benchmark ---- */
enum tbs_kernel_id { TBS_K_JOINER = 0, TBS_K_EXPAND = 1, TBS_K_SELECT = 2, TBS_K_PREDICTOR = 3,
                     TBS_K_PREP = 4, TBS_K_GEMM = 5,
                     TBS_K_ROUND = 6,   /* expansion + select/merge as one kernel (small shapes inside tbs_decode
                                           and tbs_push_segment; timing TBS_K_EXPAND or TBS_K_SELECT keeps them apart) */
                     TBS_K_COUNT = 7 };
/* Bracket every launch of the chosen kernel family (-1: none) with HIP events
 * on the context's stream. */
int tbs_profile_select(tbs_ctx *ctx, int32_t kernel_id);
/* Resolve the events recorded so far: launches, their summed duration, and
 * the summed work units (joiner, expand, prep: rows; TBS_K_GEMM, every launch of the bf16/fp32
 * GEMM kernel, joiner and predictor alike: multiply-adds M*N*K; others: hypotheses). Resets. */
int tbs_profile_read(tbs_ctx *ctx, int64_t *launches, double *total_ms, int64_t *units);
/* What the event pair itself adds: the same bracket around n launches of a kernel that does
 * nothing (k_empty, one wave), average in microseconds (HOST).  A kernel trace of the same run
 * shows k_empty's own duration; the difference is the cost events add to every bracket. */
int tbs_profile_overhead(tbs_ctx *ctx, int32_t n, double *avg_us);

const char *tbs_strerror(int code);
int tbs_last_hip_error(const tbs_ctx *ctx);

/* Plain bf16 GEMM of the joiner's own kernels, C[M,N] = A[M,K] * B[N,K]^T +
 * bias[N] with float32 accumulation and output, exported so that the MFMA
 * tilings can be checked and timed on their own.  All pointers DEVICE, row-major,
 * K a multiple of 8.  kernel: 0 = the choice the decode makes for this size;
 * 1, 2, 3 = 64x64, 128x128, 256x256 workgroup tiles of the persistent kernel;
 * 4 = the multi-stage kernel for small problems (K a multiple of 128, else
 * TBS_EINVAL).  Asynchronous on `stream`. */
int tbs_gemm_bf16(const void *A, const void *B, const float *bias, float *C, int32_t M, int32_t N,
                  int32_t K, int32_t kernel, void *stream);

#ifdef __cplusplus
}
#endif
#endif
