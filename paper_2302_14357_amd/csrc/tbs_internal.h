// Internal declarations shared by the host code and the kernel files of libtbs.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tbs.h"

typedef unsigned long long u64;
typedef uint16_t bf16_t;  // raw bf16 bit pattern

// Group A (hypotheses still emitting in this segment), structure of arrays, [U, N].
struct AView {
    int *count;     // [U]
    double *logs;   // log score
    int *node;      // trie node of the token sequence
    u64 *hash;      // hash of the token sequence
    int *len;       // number of tokens
    int *slot;      // predictor-state slot of this hypothesis
    int *pslot;     // slot of the hypothesis it was made from (source of the recurrent state)
    int *pnode;     // trie node of the hypothesis it was made from
    int *token;     // last token (-1 for hypotheses carried into the segment)
    float *dhat;    // [U, N, S] frame distribution of the last token, normalised, as natural logarithms
};

// Group B (hypotheses that took their blank for this segment), [U, BCAP].
struct BView {
    int *count;
    double *logs;
    int *node;
    u64 *hash;
    int *len;
    int *slot;
};

// Row/pair lists of the current round.
struct RowView {
    int *utt_pair0;  // [U]  first pair of each utterance
    int *utt_row0;   // [U]  first joiner row of each utterance
    int *utt_sp;     // [U]  frames of each utterance in this segment (0 = finished)
    int *utt_par;    // [U]  which of the two state arenas the utterance's current segment writes to; flips each
                     //      time the utterance starts a segment (survivors sit in the other one)
    int *pair_u, *pair_h, *pair_row0, *pair_len;  // [pairs]
    int *pair_slot;  // [pairs] predictor-state slot of the pair's hypothesis
    int *pair_pslot; // [pairs] slot of the hypothesis it was made from (source of the recurrent state)
    int *pair_frame0; // [pairs] row in enc_proj of the pair's first frame of the segment
    int *pair_tok;   // [pairs] last token of the pair's hypothesis (-1 if carried into the segment)
    int *row_enc;    // [rows] frame row in enc_proj
    int *row_slot;   // [rows] predictor-state slot
    int *counts;     // [8]: 0 pairs, 1 rows, 2 trie nodes used, 3 error flags, 4 live utterances,
                     //      5 frames joined (sum of S' over live utterances), 6 number of the launch that
                     //      published the figures (host mirror), 7 the other slot of 2 (they alternate),
                     //      8 and 9 running sums of 4 and 5 over the row lists made since the batch began
                     //      (joiner invocations and frames joined, per utterance summed)
};

enum { TBS_CNT_PAIRS = 0, TBS_CNT_ROWS = 1, TBS_CNT_NODES = 2, TBS_CNT_ERR = 3, TBS_CNT_UTTS = 4, TBS_CNT_FRAMES = 5,
       TBS_CNT_SEQ = 6, TBS_CNT_NODE_BASE = 7, TBS_CNT_ACC_CALLS = 8, TBS_CNT_ACC_JOINED = 9, TBS_CNT_SIZE = 10 };
enum { TBS_ERRF_BCAP = 1, TBS_ERRF_NODES = 2 };

// Slot layout of small shapes: hypothesis i of utterance u is pair j = u*N + i whether or not it
// exists, its frames are the joiner rows j*S .. j*S + S' - 1.  Nothing depends on the other utterances'
// counts, so no kernel has to sum them: the kernel that makes a list A also writes the descriptors of
// its pairs, takes trie nodes from the utterance's own range and tells the host its count.
struct FixedView {
    int on;
    int seg;
    const int *utt_off;   // [U] first frame row of each utterance
    int *fig;             // [U, 8] what a round needs to know of an utterance before it can start, side by side so
                          //        that one request brings all of it (indices TBS_FIG_*): S' of the segment, the
                          //        hypotheses in A, the entries of B, the state arena, then the trie nodes the
                          //        utterance has taken from its range, the range's size and its first node (the
                          //        ranges share the trie in proportion to the utterances' lengths)
    int *live_sum;        // [2] hypotheses made by all utterances in launch seq (slot seq & 1): kernels queued
                          //     behind it leave at once when it is zero
    int *host_live;       // pinned [2, U], half seq & 1: (seq << 8) | (trie full << 6) | hypotheses made
    int seq;
    const float *pool_h;  // first LSTM layer's h by state slot, and where the new hypotheses' input rows go:
    bf16_t *xh;           // xh[j, :] = bf16(h of the parent of pair j)   (null: not wanted)
    // head of a segment only: where the joiner input rows of the survivors go (null: a kernel of its own
    // makes them), the projected encoder frames and the joiner activation
    bf16_t *amat;
    const bf16_t *enc;
    int act;
    int parts;            // workgroups per utterance of the kernel that starts a segment (0 = 1)
    int xcd_rows;         // round kernel: not 0 = joiner rows per XCD (workgroup b runs on XCD b % 8 and takes an
                          // utterance whose first row lies in that XCD's range; see PartEp)
};
#define TBS_FIXED_SMAX 5   // longest segment the slot layout serves

enum { TBS_FIG_SP = 0, TBS_FIG_CNT = 1, TBS_FIG_NB = 2, TBS_FIG_PAR = 3, TBS_FIG_USED = 4, TBS_FIG_CAP = 5,
       TBS_FIG_BASE = 6, TBS_FIG_SIZE = 8 };

struct Dims {
    int U, N, S, V, Dj, blank;
    int R;      // rounds capacity
    int BCAP;   // entries of B per utterance
    int E, H, L;
    int max_nodes;
};

__host__ __device__ inline int tbs_slot_id(int u, int parity, int r, int i, int R, int N) {
    return ((u * 2 + parity) * (R + 1) + r) * N + i;
}

// Joiner activation of the bf16 path.  tanh x = 1 - 2 / (exp(2x) + 1) with the hardware exponential
// and reciprocal: the absolute error is a few fp32 units of 1, far below the bf16 rounding the
// result goes through; both kernels that form joiner input rows use it, so they agree bit for bit.
__device__ __forceinline__ float tbs_joiner_act(float x, int act) {
    if (act != 0) return fmaxf(x, 0.f);
    const float t = __expf(2.f * x);
    return 1.f - 2.f * __builtin_amdgcn_rcpf(t + 1.f);
}

// LSTM cell update done in the epilogue of the gate GEMM (small problems): the weight rows are
// stored gate-interleaved (row 4j+g = gate g of hidden unit j, gate order i, f, g, o), so a 64-wide
// output tile holds all four gates of 16 units.
struct LstmEp {
    const int *pslot, *slot, *tok;   // per row: parent's state slot, own state slot, last token
    const float *emb_gates;          // [V, 4H] gate-interleaved input half of the gates (+ bias), or null
    const float *c_par;              // cell states of this layer, indexed by slot
    float *c_new, *h_new;            // the same pools, written at the row's own slot
    const float *h_par_next;         // hidden states of the next layer (null for the last layer)
    bf16_t *out16;                   // last layer: [rows, H] top hidden state; else [rows, 2H] next layer's input
    int H;
};

// Joiner input rows made in the epilogue of the predictor projection (small problems): row r of
// the product is the projection of pair r, whose frames pair_frame0[r] .. + pair_len[r] - 1 give
// the joiner rows pair_row0[r] ..: amat[row, :] = act(enc[frame, :] + projection).
struct JoinEp {
    const int *pair_row0, *pair_len, *pair_frame0;
    const bf16_t *enc;   // [frames, Dj]
    bf16_t *amat;        // [rows, Dj]
    int act;             // 0 tanh, 1 relu
    int fgroups;         // workgroups per tile (0 = 1): each computes the tile and forms the joiner input rows of
                         // the frames t = its number, + fgroups, ...; the first also stores the projection
};

// Segments of one frame (the standard breadth-first search, Eq. 1): the joiner GEMM keeps no logits.
// Its epilogue leaves, per row and per tile of 64 columns, what the expansion of a one-frame segment
// needs of them: part[(row * tiles_n + tile) * PW ..] = maximum, sum of exp(l - maximum), the blank
// logit (-inf if blank is in another tile), a spare, then the NP largest non-blank logits in
// descending order (-inf where there are fewer) and their tokens (as integer bit patterns, -1).
struct PartEp {
    float *part;
    int np;      // NP = beam size
    int blank;
    int pieces;     // 1: the partials of a tile's four 16-column pieces go out as they are (four partials per
                    // tile, in column order), for a reader that has a lane for each; 0: merged into one
    int xcd_rows;   // (also for the joiner GEMM that stores logits) not 0: every XCD computes a range of rows
                    // of its own, all their columns, so that the logits or partials of an utterance lie in
                    // the L2 of the XCD whose workgroup of the round kernel reads them (see FixedView)
};
__host__ __device__ inline int part_width(int np) { return (4 + 2 * np + 3) & ~3; }   // (whole 16-byte pieces)

// ---- launchers (each enqueues on `st` and returns the HIP status) ----
hipError_t launch_init_batch(hipStream_t st, const Dims &d, BView B, AView A0, AView A1, RowView rv, int2 *nodes,
                             float *pool_p, float *pool_h, float *pool_c, const float *pred_init,
                             long pool_rows);
hipError_t launch_segment_begin(hipStream_t st, const Dims &d, int seg, const int *utt_T, BView B,
                                AView A, RowView rv, float *pool_p, float *pool_h, float *pool_c, long pool_rows,
                                const FixedView *fx = nullptr);
// joiner input rows in the slot layout: every row j*S + t with t < pair_len[j]
// the same by pairs (bf16; the pair count is read from the row lists' counts in device memory)
hipError_t launch_joiner_prep_pairs(hipStream_t st, const Dims &d, int act, const bf16_t *enc, const float *pool_p,
                                    RowView rv, bf16_t *amat);
hipError_t launch_joiner_prep_fixed(hipStream_t st, const Dims &d, int act, const bf16_t *enc, const float *pool_p,
                                    RowView rv, bf16_t *amat);
// gather_h / gather_xh not null: also writes gather_xh[pair, :] = bf16(gather_h[parent slot, :]) (H wide)
hipError_t launch_rowfill(hipStream_t st, const Dims &d, int seg, const int *utt_off, AView A, RowView rv,
                          int2 *nodes, int assign_nodes, int *host_counts, int seq, const float *gather_h = nullptr,
                          bf16_t *gather_xh = nullptr);
// row_begin (bf16 only, with rows_dev): only the rows [*row_begin, *rows_dev), `rows` sizing the launch
hipError_t launch_joiner_prep(hipStream_t st, const Dims &d, int dtype, int act, int rows, const void *enc,
                              const float *pool_p, RowView rv, void *amat, const int *rows_dev = nullptr,
                              const int *row_begin = nullptr);
hipError_t launch_gemm_f32(hipStream_t st, const float *A, const float *B, const float *bias, float *C, int M, int N,
                           int K, const int *out_row, long ldc);
// m_dev (launch_gemm_bf16 only where gemm_small_fits; the fused forms always): the launch is enqueued
// before the host knows the row count; M is an upper bound and the count is read from *m_dev
hipError_t launch_gemm_bf16(hipStream_t st, const bf16_t *A, const bf16_t *B, const float *bias, float *C, int M,
                            int N, int K, const int *out_row, long ldc, int kernel = 0, const int *m_dev = nullptr,
                            bool xcd_rows = false);
// rows per XCD when k_gemm_small gives every XCD a row range of its own (PartEp::xcd_rows)
inline int gemm_small_xcd_rows(int M) { return 64 * ((((M + 63) / 64) + 7) / 8); }
hipError_t launch_gemm_bf16_rows(hipStream_t st, const bf16_t *A, const bf16_t *B, const float *bias, float *C,
                                 int m_max, int N, int K, long ldc, const int *m_begin, const int *m_end);
#define GS_TILES 320          // tiles of 64 x 64 up to which the small-problem GEMM kernel is chosen by size
#define GS_TILES_FIXED 1024   // the same for the slot layout (measured on the Librispeech-like shape: 96 to 256
                              // utterances decode 5-16 % faster in it than with row lists, 320 the same)
bool gemm_small_fits(int M, int N, int K, int max_tiles = GS_TILES);
// true if launch_gemm_lstm can run this problem (small, K a multiple of 128 that fits the LDS stages)
bool gemm_lstm_fits(int M, int H, int K, int max_tiles = GS_TILES);
// any_dev (both fused forms): rows may be dead (state slot < 0) anywhere, and if *any_dev is zero
// the whole launch leaves at once
hipError_t launch_gemm_lstm(hipStream_t st, const bf16_t *A, const bf16_t *Wp, const float *biasp, int M, int K,
                            const LstmEp &ep, const int *m_dev = nullptr, const int *any_dev = nullptr);
// the same for the projection GEMM that also makes the next joiner call's input rows (bf16 models)
bool gemm_join_fits(int M, int N, int K, int max_tiles = GS_TILES);
hipError_t launch_gemm_join(hipStream_t st, const bf16_t *A, const bf16_t *B, const float *bias, float *C, int M,
                            int N, int K, const int *out_row, long ldc, const JoinEp &jp, const int *m_dev = nullptr,
                            const int *any_dev = nullptr);
// joiner GEMM of one-frame segments: row partials instead of logits (see PartEp)
bool gemm_part_fits(int M, int N, int K, int np, int max_tiles = GS_TILES);
hipError_t launch_gemm_part(hipStream_t st, const bf16_t *A, const bf16_t *B, const float *bias, int M, int N, int K,
                            const PartEp &pe);
hipError_t launch_permute_gate_rows(hipStream_t st, const void *src, void *dst, int H, long row_bytes);
hipError_t launch_expand(hipStream_t st, const Dims &d, int pairs, const float *logits, AView A, RowView rv,
                         float *row_lc, float *dphi, float *cand_score, int *cand_tok, float *row_stats,
                         float *delta_nb, int force_generic, const int *pairs_dev = nullptr, int pair_base = 0);
hipError_t launch_select_merge(hipStream_t st, const Dims &d, int round, int drop, const float *logits,
                               const float *row_lc, const float *dphi, const float *cand_score,
                               const int *cand_tok, AView A, AView An, BView B, RowView rv, const int2 *nodes);
// expansion and select/merge of a round in one kernel, a workgroup per utterance (small shapes:
// round_fits says whether the shape is served)
bool round_fits(const Dims &d);
hipError_t launch_round(hipStream_t st, const Dims &d, int round, int drop, const float *logits, AView A, AView An,
                        BView B, RowView rv, int2 *nodes, float *row_stats, float *delta_nb,
                        const FixedView *fx = nullptr);
// the same for one-frame segments in the slot layout, from the joiner GEMM's row partials
bool round_s1_fits(const Dims &d);
// (tiles_n: partials per row, in column order: the vocabulary's 64-column tiles, or their 16-column pieces)
hipError_t launch_round_s1(hipStream_t st, const Dims &d, int round, int drop, const float *part, int tiles_n, AView A,
                           AView An, BView B, RowView rv, int2 *nodes, const FixedView *fx);
hipError_t launch_pred_gather(hipStream_t st, const Dims &d, int dtype, int pairs, AView A, RowView rv,
                              const void *embed, const float *pool_h, void *xh);
hipError_t launch_pred_gather_h(hipStream_t st, const Dims &d, int pairs, AView A, RowView rv, const float *pool_h,
                                bf16_t *xh);
hipError_t launch_lstm_pointwise(hipStream_t st, const Dims &d, int dtype, int pairs, int layer, AView A, RowView rv,
                                 const float *gates, float *pool_h, float *pool_c, long pool_rows, void *xh_next,
                                 void *htop, const float *emb_gates);
hipError_t launch_finalize(hipStream_t st, const Dims &d, BView B, const int2 *nodes, int *res_count, int *res_len,
                           double *res_logs, int *res_tok, int max_len);
hipError_t launch_hyps_dump(hipStream_t st, const Dims &d, int group, AView A, BView B, const int2 *nodes, int cap,
                            int max_len, int *tok, int *len, double *logs, int *count);
hipError_t launch_gather_pred(hipStream_t st, const Dims &d, AView A, const float *pool_p, float *out, int scatter);
hipError_t launch_concat_weights(hipStream_t st, int elem_bytes, const void *w_ih, const void *w_hh, void *wcat,
                                 int rows, int in_dim, int hid);
hipError_t launch_debug_fill_a(hipStream_t st, const Dims &d, AView A);
// rows of row_bytes bytes: for every utterance u, n[u] rows from src row src_row[u] on to dst row
// dst_row[u] on (desc = [src_row | dst_row | n], each [U]); the ranges of src and dst must not overlap
hipError_t launch_stream_copy(hipStream_t st, int U, const void *src, void *dst, const int *desc, long row_bytes);
hipError_t launch_empty(hipStream_t st);   // a kernel that does nothing (timing yardstick)
hipError_t launch_set_sp(hipStream_t st, const Dims &d, int seg, const int *utt_T, RowView rv);
