// Host side of libtbs: context, workspaces, the C ABI of include/tbs.h and the
// lock-step driver of Algorithm 1 (outer loop over segments, inner loop over
// token-emission rounds).  All arithmetic of the method runs in the kernels of
// the other files; this file only sizes buffers, orders launches and moves
// counts and results between device and host.
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "tbs_internal.h"
#include <math.h>


namespace {

enum State { ST_INIT = 0, ST_BEGUN, ST_READY, ST_JOINED, ST_EXPANDED, ST_SELECTED };

struct EventPair {
    hipEvent_t a, b;
};

}  // namespace

struct tbs_ctx {
    tbs_config cfg;
    tbs_weights w;
    hipStream_t stream;
    Dims d;       // capacities (U = max_utts)
    Dims cur;     // current batch (U = bound utterances)
    int state;
    int last_hip;
    std::vector<void *> allocs;

    // batch
    const void *enc;
    int *utt_T, *utt_off;
    std::vector<int> h_T;
    int max_T;
    int seg, round, a_cur;

    AView A[2];
    BView B;
    RowView rv;
    // streaming: per-utterance frame buffers [U, stream_cap, Dj], a spare area [U, S, Dj] for moving
    // leftovers to the front, and what the host knows of them
    void *stream_enc, *stream_tmp;
    int stream_cap;
    bool streaming;
    std::vector<int> s_fill;   // frames buffered per utterance (they start at the front of its buffer)
    int *h_desc;               // pinned: descriptors of the frame copies and of a decode step
    int *d_desc;
    int *h_counts;      // pinned host mirror of rv.counts
    int *h_counts_dev;  // device view of the same memory
    int seq;            // number of the last scan asked to publish its counts there
    bool prep_ahead;    // the joiner input rows of the coming call are already being made (see tbs_segment_begin)
    int pred_ahead;     // predictor kernels of this round already enqueued (see tbs_select_merge): 1 the LSTM layers, 2 all
    bool join_ahead;    // and so is the joiner GEMM of the next round
    bool expanded_ahead; // tbs_joiner_segment already ran the expansion, piece by piece behind the GEMM of each piece
    // slot layout (small shapes inside tbs_decode / tbs_push_segment, see FixedView)
    bool fixed;         // the current batch runs in the slot layout
    bool s1;            // ... with segments of one frame and no logits (the joiner GEMM keeps row partials)
    float *part;        // [U*N, tiles of 64 columns, part_width(N)] row partials (seg_s = 1 only)
    int *utt_fig;       // [U, TBS_FIG_SIZE] each utterance's figures for the round kernel, among them its range of the trie
    int *live_sum;      // [2] hypotheses made per launch, alternating
    int *h_live;        // pinned [U]: what each utterance's workgroup tells the host
    int *h_live_dev;    // device view of the same memory
    std::vector<int> live_u;   // hypotheses each utterance takes into the coming round
    int64_t fx_calls, fx_joined;   // joiner invocations and frames joined, counted on the host in this layout
    int2 *nodes;
    long pool_rows;
    float *pool_p, *pool_h, *pool_c;

    void *amat;
    float *logits, *row_lc, *row_stats, *dphi, *delta_nb, *cand_score;
    int *cand_tok;

    void *wcat[TBS_MAX_LAYERS];
    float *emb_gates;   // bf16 models: [V, 4H] = embed * W_ih(layer 0)^T + b(layer 0)
    // gate-interleaved copies (row 4j+g = gate g of unit j) for the GEMM that updates the cell in its
    // epilogue: layer 0 [4H, H] (recurrent half), layers >= 1 [4H, 2H]; biases of layers >= 1; the table
    void *wperm[TBS_MAX_LAYERS];
    float *bperm[TBS_MAX_LAYERS];
    float *emb_gates_perm;
    void *xh[2];
    void *htop;
    float *gates;

    // results
    int *res_count, *res_len, *res_tok;
    double *res_logs;
    int res_max_len;

    // counters
    int64_t n_frames, n_launches;   // (joiner invocations and frames joined are counted on the device)

    // profiling
    int prof_kernel;
    std::vector<EventPair> events;
    size_t ev_used;
    int64_t prof_units;
};

// Scratch of tbs_debug_hyps_noalloc: one array per GPU the library is loaded on, held until the
// process ends.  In host code the array's name is only a stand-in for the symbol, not a device
// address: the address on a device is asked for once per device, with that device current (each GPU
// has its own copy at its own address), and only that pointer is handed to kernels and copies.
#define TBS_NOALLOC_BYTES (2u << 20)
#define TBS_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[TBS_NOALLOC_BYTES];
static void *g_scratch_ptr[TBS_MAX_DEVICES];
static std::mutex g_scratch_mutex;

// (the caller has made `device` current)
static hipError_t scratch_resolve(int device) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return hipSuccess;
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = p;
    return hipSuccess;
}

#define HIPCHK(ctx, expr)                       \
    do {                                        \
        hipError_t e_ = (expr);                 \
        if (e_ != hipSuccess) {                 \
            (ctx)->last_hip = (int)e_;          \
            return TBS_EHIP;                    \
        }                                       \
    } while (0)

namespace {

template <typename T>
int dev_alloc(tbs_ctx *c, T **p, size_t n) {
    void *q = nullptr;
    size_t bytes = std::max<size_t>(n, 1) * sizeof(T);
    hipError_t e = hipMalloc(&q, bytes);
    if (e != hipSuccess) {
        c->last_hip = (int)e;
        (void)hipGetLastError();
        return TBS_ENOMEM;
    }
    c->allocs.push_back(q);
    *p = (T *)q;
    return TBS_OK;
}

int alloc_aview(tbs_ctx *c, AView *a, long UN, int S, int U) {
    int rc = 0;
    rc |= dev_alloc(c, &a->count, U);
    rc |= dev_alloc(c, &a->logs, UN);
    rc |= dev_alloc(c, &a->node, UN);
    rc |= dev_alloc(c, &a->hash, UN);
    rc |= dev_alloc(c, &a->len, UN);
    rc |= dev_alloc(c, &a->slot, UN);
    rc |= dev_alloc(c, &a->pslot, UN);
    rc |= dev_alloc(c, &a->pnode, UN);
    rc |= dev_alloc(c, &a->token, UN);
    rc |= dev_alloc(c, &a->dhat, UN * S);
    return rc ? TBS_ENOMEM : TBS_OK;
}

struct ProfScope {
    tbs_ctx *c;
    bool on;
    size_t idx;
    ProfScope(tbs_ctx *ctx, int kernel, int64_t units) : c(ctx), on(false), idx(0) {
        if (c->prof_kernel == kernel && c->ev_used < c->events.size()) {
            on = true;
            idx = c->ev_used++;
            c->prof_units += units;
            (void)hipEventRecord(c->events[idx].a, c->stream);
        }
    }
    ~ProfScope() {
        if (on) (void)hipEventRecord(c->events[idx].b, c->stream);
    }
};

// Wait for the counts of the scan numbered c->seq without draining the stream: the kernel that
// runs the scan writes them into pinned host memory and its number last, so the host can size
// and enqueue the next launches while the kernels behind that scan are still running.
// The wait is bounded on the host: a stream that ends without the number, a stream error, or
// TBS_WAIT_LIMIT_S seconds without it (no kernel of this library runs anywhere near that long)
// all come back as an error code instead of a call that never returns.
#define TBS_WAIT_LIMIT_S 20
hipError_t wait_counts(tbs_ctx *c) {
    const int want = c->seq;
    std::chrono::steady_clock::time_point t0;
    bool timing = false;
    for (unsigned spin = 1;; ++spin) {
        if (__atomic_load_n(&c->h_counts[TBS_CNT_SEQ], __ATOMIC_ACQUIRE) == want) return hipSuccess;
        if ((spin & 0x3FFFFF) == 0) {   // every few milliseconds (a query costs microseconds, during which the
                                        // number would go unnoticed): has the stream failed, or ended without it?
            const hipError_t e = hipStreamQuery(c->stream);
            if (e == hipSuccess)
                return __atomic_load_n(&c->h_counts[TBS_CNT_SEQ], __ATOMIC_ACQUIRE) == want ? hipSuccess
                                                                                              : hipErrorUnknown;
            if (e != hipErrorNotReady) return e;
            const auto now = std::chrono::steady_clock::now();
            if (!timing) {
                t0 = now;
                timing = true;
            } else if (now - t0 > std::chrono::seconds(TBS_WAIT_LIMIT_S)) {
                return hipErrorLaunchTimeOut;
            }
        }
    }
}

int check_err_flags(tbs_ctx *c) {
    int err = c->h_counts[TBS_CNT_ERR];
    if (err) return TBS_EOVERFLOW;
    return TBS_OK;
}

int elem_bytes(const tbs_ctx *c) { return c->cfg.dtype == 1 ? 2 : 4; }

hipError_t gemm(tbs_ctx *c, const void *A, const void *B, const float *bias, float *C, int M, int N, int K,
                const int *out_row, long ldc) {
    ProfScope ps(c, TBS_K_GEMM, (int64_t)M * N * K);
    if (c->cfg.dtype == 1)
        return launch_gemm_bf16(c->stream, (const bf16_t *)A, (const bf16_t *)B, bias, C, M, N, K, out_row, ldc);
    return launch_gemm_f32(c->stream, (const float *)A, (const float *)B, bias, C, M, N, K, out_row, ldc);
}

}  // namespace

extern "C" {

const char *tbs_strerror(int code) {
    switch (code) {
        case TBS_OK: return "ok";
        case TBS_EINVAL: return "invalid argument or unsupported shape";
        case TBS_ESTATE: return "call out of order";
        case TBS_ENOMEM: return "allocation failed";
        case TBS_EHIP: return "HIP call failed";
        case TBS_EOVERFLOW: return "capacity exceeded (rounds per segment, merged list, trie nodes or max_len)";
        case TBS_ELIMIT: return "request larger than the fixed scratch of an entry point that does not allocate";
        default: return "unknown error";
    }
}

int tbs_last_hip_error(const tbs_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

void tbs_free(tbs_ctx *c) {
    if (!c) return;
    (void)hipSetDevice(c->cfg.device_id);
    (void)hipStreamSynchronize(c->stream);
    for (void *p : c->allocs) (void)hipFree(p);
    if (c->h_counts) (void)hipHostFree(c->h_counts);
    if (c->h_live) (void)hipHostFree(c->h_live);
    if (c->h_desc) (void)hipHostFree(c->h_desc);
    for (auto &e : c->events) {
        (void)hipEventDestroy(e.a);
        (void)hipEventDestroy(e.b);
    }
    delete c;
}

int tbs_init(const tbs_config *cfg, const tbs_weights *w, tbs_ctx **out) {
    if (!cfg || !w || !out) return TBS_EINVAL;
    *out = nullptr;
    if (cfg->d_joint < 1 || cfg->vocab < 2 || cfg->blank_id < 0 || cfg->blank_id >= cfg->vocab) return TBS_EINVAL;
    if (cfg->beam_n < 1 || cfg->beam_n > TBS_MAX_BEAM || cfg->seg_s < 1 || cfg->seg_s > TBS_MAX_SEG)
        return TBS_EINVAL;
    if (cfg->max_utts < 1 || cfg->max_frames_total < 0) return TBS_EINVAL;
    if (cfg->device_id < 0 || cfg->device_id >= TBS_MAX_DEVICES) return TBS_EINVAL;
    if (cfg->pred_layers < 1 || cfg->pred_layers > TBS_MAX_LAYERS || cfg->pred_hidden < 1 || cfg->pred_embed < 1)
        return TBS_EINVAL;
    if (cfg->act < 0 || cfg->act > 1 || cfg->dtype < 0 || cfg->dtype > 1) return TBS_EINVAL;
    if (cfg->max_rounds_per_segment < 0 || cfg->rounds_capacity < 0 || cfg->max_nodes < 0) return TBS_EINVAL;
    if (cfg->max_result_len < 0) return TBS_EINVAL;
    if (cfg->joiner_chunk_rows < 0) return TBS_EINVAL;
    if (cfg->stream_buffer_frames < 0 || (cfg->stream_buffer_frames != 0 && cfg->stream_buffer_frames < cfg->seg_s))
        return TBS_EINVAL;
    if (cfg->vocab > 16000) return TBS_EINVAL;  // the expansion kernel keeps one row of scores in LDS
    if (cfg->dtype == 1 && (cfg->d_joint % 8 || cfg->pred_hidden % 8 || cfg->pred_embed % 8)) return TBS_EINVAL;
    if (!w->w_out || !w->b_out || !w->embed || !w->w_proj || !w->b_proj || !w->pred_init) return TBS_EINVAL;
    for (int l = 0; l < cfg->pred_layers; ++l)
        if (!w->w_ih[l] || !w->w_hh[l] || !w->b_lstm[l]) return TBS_EINVAL;

    tbs_ctx *c = new (std::nothrow) tbs_ctx();
    if (!c) return TBS_ENOMEM;
    c->cfg = *cfg;
    c->w = *w;
    c->stream = (hipStream_t)cfg->stream;
    c->state = ST_INIT;
    c->last_hip = 0;
    c->h_counts = nullptr;
    c->h_live = nullptr;
    c->fixed = false;
    c->h_desc = nullptr;
    c->d_desc = nullptr;
    c->stream_enc = c->stream_tmp = nullptr;
    c->stream_cap = 0;
    c->streaming = false;
    c->res_tok = nullptr;
    c->res_max_len = 0;
    c->prof_kernel = -1;
    c->ev_used = 0;
    c->prof_units = 0;
    hipError_t e = hipSetDevice(cfg->device_id);
    if (e == hipSuccess) e = scratch_resolve(cfg->device_id);   // this device's address of the static scratch
    if (e != hipSuccess) {
        c->last_hip = (int)e;
        delete c;
        return TBS_EHIP;
    }

    Dims &d = c->d;
    d.U = cfg->max_utts;
    d.N = cfg->beam_n;
    d.S = cfg->seg_s;
    d.V = cfg->vocab;
    d.Dj = cfg->d_joint;
    d.blank = cfg->blank_id;
    d.R = cfg->rounds_capacity > 0 ? cfg->rounds_capacity : 32;
    if (cfg->max_rounds_per_segment > 0) d.R = cfg->max_rounds_per_segment;
    d.BCAP = d.N * d.R;
    if (d.BCAP > 2048) {   // the merge kernel stages one utterance's B list in LDS
        delete c;
        return TBS_EINVAL;
    }
    d.E = cfg->pred_embed;
    d.H = cfg->pred_hidden;
    d.L = cfg->pred_layers;
    long dn = cfg->max_nodes > 0 ? (long)cfg->max_nodes
                                 : 4L * d.N * ((long)cfg->max_frames_total + (long)d.U * d.S) + 16;
    if (dn > 2000000000L) dn = 2000000000L;
    d.max_nodes = (int)dn;

    const long U = d.U, UN = U * d.N, M = UN * d.S;
    int rc = 0;
    rc |= alloc_aview(c, &c->A[0], UN, d.S, d.U);
    rc |= alloc_aview(c, &c->A[1], UN, d.S, d.U);
    rc |= dev_alloc(c, &c->B.count, U);
    rc |= dev_alloc(c, &c->B.logs, U * d.BCAP);
    rc |= dev_alloc(c, &c->B.node, U * d.BCAP);
    rc |= dev_alloc(c, &c->B.hash, U * d.BCAP);
    rc |= dev_alloc(c, &c->B.len, U * d.BCAP);
    rc |= dev_alloc(c, &c->B.slot, U * d.BCAP);
    rc |= dev_alloc(c, &c->rv.utt_pair0, U);
    rc |= dev_alloc(c, &c->rv.utt_row0, U);
    rc |= dev_alloc(c, &c->rv.pair_slot, UN);
    rc |= dev_alloc(c, &c->rv.pair_pslot, UN);
    rc |= dev_alloc(c, &c->rv.pair_frame0, UN);
    rc |= dev_alloc(c, &c->rv.pair_tok, UN);
    rc |= dev_alloc(c, &c->rv.utt_sp, U);
    rc |= dev_alloc(c, &c->rv.utt_par, U);
    rc |= dev_alloc(c, &c->rv.pair_u, UN);
    rc |= dev_alloc(c, &c->rv.pair_h, UN);
    rc |= dev_alloc(c, &c->rv.pair_row0, UN);
    rc |= dev_alloc(c, &c->rv.pair_len, UN);
    rc |= dev_alloc(c, &c->rv.row_enc, M);
    rc |= dev_alloc(c, &c->rv.row_slot, M);
    rc |= dev_alloc(c, &c->rv.counts, TBS_CNT_SIZE);
    rc |= dev_alloc(c, &c->utt_fig, U * TBS_FIG_SIZE);
    rc |= dev_alloc(c, &c->live_sum, 2);
    // (utterance lengths, first frames and the frame-copy descriptors of a push side by side, so that
    // one copy from pinned memory brings all a push has to tell the kernels)
    rc |= dev_alloc(c, &c->utt_T, 5 * (size_t)U + 1);
    if (rc == 0) {
        c->utt_off = c->utt_T + U;
        c->d_desc = c->utt_off + U + 1;
    }
    rc |= dev_alloc(c, &c->nodes, (size_t)d.max_nodes);
    c->pool_rows = U * 2 * (d.R + 1) * d.N;
    rc |= dev_alloc(c, &c->pool_p, (size_t)c->pool_rows * d.Dj);
    rc |= dev_alloc(c, &c->pool_h, (size_t)c->pool_rows * d.H * d.L);
    rc |= dev_alloc(c, &c->pool_c, (size_t)c->pool_rows * d.H * d.L);
    {
        char *p = nullptr;
        rc |= dev_alloc(c, &p, (size_t)M * d.Dj * elem_bytes(c));
        c->amat = p;
    }
    rc |= dev_alloc(c, &c->logits, (size_t)M * d.V);
    c->part = nullptr;
    // (room for a partial per 16-column piece where the round kernel has a lane for each, else per 64-column tile)
    if (d.S == 1 && cfg->dtype == 1)
        rc |= dev_alloc(c, &c->part, UN * (size_t)((d.V + 63) / 64) * ((d.V + 63) / 64 <= 16 ? 4 : 1) * part_width(d.N));
    rc |= dev_alloc(c, &c->row_lc, M);
    rc |= dev_alloc(c, &c->dphi, UN);
    rc |= dev_alloc(c, &c->cand_score, UN * d.N);
    rc |= dev_alloc(c, &c->cand_tok, UN * d.N);
    c->row_stats = nullptr;
    c->delta_nb = nullptr;
    if (cfg->debug & 1) {
        rc |= dev_alloc(c, &c->row_stats, (size_t)M * 3);
        rc |= dev_alloc(c, &c->delta_nb, (size_t)UN * d.V);
    }
    const int xw = std::max(d.E + d.H, 2 * d.H);
    for (int i = 0; i < 2; ++i) {
        char *p = nullptr;
        rc |= dev_alloc(c, &p, (size_t)UN * xw * elem_bytes(c));
        c->xh[i] = p;
    }
    {
        char *p = nullptr;
        rc |= dev_alloc(c, &p, (size_t)UN * d.H * elem_bytes(c));
        c->htop = p;
    }
    rc |= dev_alloc(c, &c->gates, (size_t)UN * 4 * d.H);
    for (int l = 0; l < d.L; ++l) {
        int in_dim = l == 0 ? d.E : d.H;
        char *p = nullptr;
        rc |= dev_alloc(c, &p, (size_t)4 * d.H * (in_dim + d.H) * elem_bytes(c));
        c->wcat[l] = p;
    }
    c->emb_gates = nullptr;
    c->emb_gates_perm = nullptr;
    char *wih0p = nullptr;      // scratch of the table's construction
    float *b0p = nullptr;
    if (cfg->dtype == 1) {
        rc |= dev_alloc(c, &c->emb_gates, (size_t)d.V * 4 * d.H);
        rc |= dev_alloc(c, &c->emb_gates_perm, (size_t)d.V * 4 * d.H);
        rc |= dev_alloc(c, &wih0p, (size_t)4 * d.H * d.E * 2);
        rc |= dev_alloc(c, &b0p, (size_t)4 * d.H);
        for (int l = 0; l < d.L; ++l) {
            char *p = nullptr;
            rc |= dev_alloc(c, &p, (size_t)4 * d.H * (l == 0 ? d.H : 2 * d.H) * 2);
            c->wperm[l] = p;
            c->bperm[l] = nullptr;
            if (l > 0) rc |= dev_alloc(c, &c->bperm[l], (size_t)4 * d.H);
        }
    }
    rc |= dev_alloc(c, &c->res_count, U);
    rc |= dev_alloc(c, &c->res_len, UN);
    rc |= dev_alloc(c, &c->res_logs, UN);
    c->res_max_len = cfg->max_result_len > 0 ? cfg->max_result_len : 256;
    rc |= dev_alloc(c, &c->res_tok, (size_t)UN * c->res_max_len);
    if (rc) {
        tbs_free(c);
        return TBS_ENOMEM;
    }
    if (cfg->stream_buffer_frames > 0) {
        c->stream_cap = cfg->stream_buffer_frames;
        char *p = nullptr, *q = nullptr;
        rc = dev_alloc(c, &p, (size_t)U * c->stream_cap * d.Dj * elem_bytes(c));
        rc |= dev_alloc(c, &q, (size_t)U * d.S * d.Dj * elem_bytes(c));
        c->stream_enc = p;
        c->stream_tmp = q;
        if (rc == 0 && hipHostMalloc((void **)&c->h_desc, (11 * (size_t)U + 1) * sizeof(int), hipHostMallocDefault) != hipSuccess) rc = 1;
        if (rc) {
            tbs_free(c);
            return TBS_ENOMEM;
        }
    }
    e = hipHostMalloc((void **)&c->h_counts, TBS_CNT_SIZE * sizeof(int), hipHostMallocMapped);
    if (e != hipSuccess) {
        c->last_hip = (int)e;
        tbs_free(c);
        return TBS_ENOMEM;
    }
    memset(c->h_counts, 0, TBS_CNT_SIZE * sizeof(int));
    e = hipHostMalloc((void **)&c->h_live, 2 * (size_t)U * sizeof(int), hipHostMallocMapped);
    if (e == hipSuccess) e = hipHostGetDevicePointer((void **)&c->h_live_dev, c->h_live, 0);
    if (e != hipSuccess) {
        c->last_hip = (int)e;
        tbs_free(c);
        return TBS_ENOMEM;
    }
    memset(c->h_live, 0, 2 * (size_t)U * sizeof(int));
    e = hipHostGetDevicePointer((void **)&c->h_counts_dev, c->h_counts, 0);
    if (e != hipSuccess) {
        c->last_hip = (int)e;
        tbs_free(c);
        return TBS_EHIP;
    }
    for (int l = 0; l < d.L; ++l) {
        int in_dim = l == 0 ? d.E : d.H;
        e = launch_concat_weights(c->stream, elem_bytes(c), w->w_ih[l], w->w_hh[l], c->wcat[l], 4 * d.H, in_dim,
                                  d.H);
        if (e != hipSuccess) {
            c->last_hip = (int)e;
            tbs_free(c);
            return TBS_EHIP;
        }
    }
    if (c->emb_gates) {
        // gate-interleaved copies: the table through the permuted input weights and bias of layer 0,
        // the recurrent (layers >= 1: concatenated) weights and biases directly
        e = launch_permute_gate_rows(c->stream, w->w_ih[0], wih0p, d.H, (long)d.E * 2);
        if (e == hipSuccess) e = launch_permute_gate_rows(c->stream, w->b_lstm[0], b0p, d.H, 4);
        if (e == hipSuccess)
            e = launch_gemm_bf16(c->stream, (const bf16_t *)w->embed, (const bf16_t *)wih0p, b0p, c->emb_gates_perm, d.V,
                                 4 * d.H, d.E, nullptr, 4L * d.H);
        for (int l = 0; l < d.L && e == hipSuccess; ++l) {
            if (l == 0) {
                e = launch_permute_gate_rows(c->stream, w->w_hh[0], c->wperm[0], d.H, (long)d.H * 2);
            } else {
                e = launch_permute_gate_rows(c->stream, c->wcat[l], c->wperm[l], d.H, (long)2 * d.H * 2);
                if (e == hipSuccess) e = launch_permute_gate_rows(c->stream, w->b_lstm[l], c->bperm[l], d.H, 4);
            }
        }
        if (e == hipSuccess)
            e = launch_gemm_bf16(c->stream, (const bf16_t *)w->embed, (const bf16_t *)w->w_ih[0], w->b_lstm[0],
                             c->emb_gates, d.V, 4 * d.H, d.E, nullptr, 4L * d.H);
        if (e != hipSuccess) {
            c->last_hip = (int)e;
            tbs_free(c);
            return TBS_EHIP;
        }
    }
    e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
        c->last_hip = (int)e;
        tbs_free(c);
        return TBS_EHIP;
    }
    c->n_frames = c->n_launches = 0;
    *out = c;
    return TBS_OK;
}

static bool predictor_all_fused(const tbs_ctx *c, int M, int max_tiles = GS_TILES);

// The slot layout serves a batch when every kernel of a round has its small-shape form: the joiner
// GEMM over all U*N*S rows in one wave of workgroups, the one-kernel expansion + select/merge, the
// LSTM layers with the cell update and the projection with the joiner input rows in their GEMMs'
// epilogues.  Debug bits that ask for any of the separate forms (or bit 8, for this layout itself)
// keep the row lists.
// Segments of one frame: the joiner GEMM can keep row partials instead of logits (unless debug output
// that needs the logits, or debug bit 9, asks for them), and the round kernel then has no limit on
// the vocabulary from its registers.  Measured on the Librispeech-like batch (ms per decode, with
// logits / without): N = 2: 25.7 / 24.6, N = 3: 26.7 / 25.6, N = 4: 27.2 / 26.7, N = 5: 28.4 / 29.0, N = 8:
// 34.0 / 37.0, N = 10: 47.0 / 47.3.  The logits of a small batch never leave the cache, and picking the N
// best of every 16 logits costs the GEMM N rounds of a 16-way arg-max: the partials serve beams up to 4,
// the vocabularies the form with logits cannot hold, and debug bit 15.
static bool one_frame_ok(const tbs_ctx *c) {
    const Dims &d = c->cur;
    if (!c->part || (c->cfg.debug & (1 | 512)) || !round_s1_fits(d) || !gemm_part_fits(d.U * d.N, d.V, d.Dj, d.N, GS_TILES_FIXED))
        return false;
    return !round_fits(d) || d.N <= 4 || (c->cfg.debug & 32768);
}

static bool fixed_layout_ok(const tbs_ctx *c) {
    const Dims &d = c->cur;
    if (c->cfg.dtype != 1 || (c->cfg.debug & (2 | 8 | 16 | 32 | 64 | 128 | 256)) || c->cfg.joiner_chunk_rows > 0)
        return false;
    if ((d.H & 3) || (long)d.max_nodes - 1 < (long)d.U) return false;
    return (round_fits(d) || one_frame_ok(c)) && gemm_small_fits(d.U * d.N * d.S, d.V, d.Dj, GS_TILES_FIXED) &&
           predictor_all_fused(c, d.U * d.N, GS_TILES_FIXED);
}

// The joiner input rows act(e + p) of the current row lists (Section 3.1), as a kernel of its own.  rows =
// their number, or with rows_dev the most there can be (the launch goes out before the host knows).
// bf16 and segments of several frames: a thread per pair and 8 columns, the pair's p read once and
// all its frames requested together (the pair count comes from the row lists' counts in device
// memory either way); otherwise a thread per row and 8 columns.
static hipError_t joiner_rows(tbs_ctx *c, int rows, const int *rows_dev) {
    if (c->cfg.dtype == 1 && c->cur.S >= 2 && !(c->cfg.debug & 8192))
        return launch_joiner_prep_pairs(c->stream, c->cur, c->cfg.act, (const bf16_t *)c->enc, c->pool_p, c->rv,
                                        (bf16_t *)c->amat);
    return launch_joiner_prep(c->stream, c->cur, c->cfg.dtype, c->cfg.act, rows, c->enc, c->pool_p, c->rv, c->amat,
                              rows_dev);
}

// B = [([], 1, InitPredictor(), Null)] for U utterances whose lengths and first frames are h_T / offsets
static int begin_batch(tbs_ctx *c, const void *enc, const int32_t *offsets, int32_t U, int max_T, long frames) {
    HIPCHK(c, hipSetDevice(c->cfg.device_id));
    c->cur = c->d;
    c->cur.U = U;
    c->enc = enc;
    c->max_T = max_T;
    HIPCHK(c, hipMemcpyAsync(c->utt_T, c->h_T.data(), sizeof(int) * U, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(c->utt_off, offsets, sizeof(int) * (U + 1), hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, launch_init_batch(c->stream, c->cur, c->B, c->A[0], c->A[1], c->rv, c->nodes, c->pool_p, c->pool_h,
                                c->pool_c, c->w.pred_init, c->pool_rows));
    HIPCHK(c, hipMemsetAsync(c->live_sum, 0, sizeof(int) * 2, c->stream));
    memset(c->h_live, 0, 2 * sizeof(int) * (size_t)c->d.U);
    c->fx_calls = c->fx_joined = 0;
    // Slot layout: every utterance takes trie nodes from a range of its own, sized in proportion to
    // its length (a stream's utterances, whose lengths are not known, share equally); node 0 is the root.
    std::vector<int> fig((size_t)U * TBS_FIG_SIZE, 0);
    {
        const int S = c->cur.S;
        double weight_all = 0.0;
        for (int u = 0; u < U; ++u) weight_all += max_T > 0 ? (double)(c->h_T[u] + S) : 1.0;
        const long pool = (long)c->cur.max_nodes - 1;
        long at = 1;
        for (int u = 0; u < U; ++u) {
            const double w = max_T > 0 ? (double)(c->h_T[u] + S) : 1.0;
            long n = (long)((double)pool * (w / weight_all));
            if (at + n > (long)c->cur.max_nodes) n = (long)c->cur.max_nodes - at;
            fig[(size_t)u * TBS_FIG_SIZE + TBS_FIG_BASE] = (int)at;
            fig[(size_t)u * TBS_FIG_SIZE + TBS_FIG_CAP] = (int)(n < 0 ? 0 : n);
            at += n < 0 ? 0 : n;
        }
    }
    HIPCHK(c, hipMemcpyAsync(c->utt_fig, fig.data(), sizeof(int) * fig.size(), hipMemcpyHostToDevice, c->stream));
    // the host arrays above are read by the copies: finish them before returning
    HIPCHK(c, hipStreamSynchronize(c->stream));
    c->seg = -1;
    c->round = 0;
    c->a_cur = 0;
    memset(c->h_counts, 0, TBS_CNT_SIZE * sizeof(int));
    c->h_counts[TBS_CNT_NODES] = 1;
    c->seq = 0;
    c->prep_ahead = false;
    c->pred_ahead = 0;
    c->join_ahead = false;
    c->expanded_ahead = false;
    c->n_launches = 0;
    c->n_frames = frames;
    c->state = ST_BEGUN;
    c->fixed = fixed_layout_ok(c);
    c->s1 = c->fixed && one_frame_ok(c);
    return TBS_OK;
}

int tbs_begin(tbs_ctx *c, const void *enc_proj, const int32_t *frame_offsets, int32_t U) {
    if (!c || !frame_offsets || U < 1 || U > c->d.U) return TBS_EINVAL;
    if (frame_offsets[0] != 0) return TBS_EINVAL;
    int max_T = 0;
    c->h_T.assign(U, 0);
    for (int u = 0; u < U; ++u) {
        int T = frame_offsets[u + 1] - frame_offsets[u];
        if (T < 0) return TBS_EINVAL;
        c->h_T[u] = T;
        max_T = std::max(max_T, T);
    }
    if (frame_offsets[U] > c->cfg.max_frames_total) return TBS_EINVAL;
    if (frame_offsets[U] > 0 && !enc_proj) return TBS_EINVAL;
    c->streaming = false;
    return begin_batch(c, enc_proj, frame_offsets, U, max_T, frame_offsets[U]);
}

int tbs_stream_begin(tbs_ctx *c, int32_t U) {
    if (!c || U < 1 || U > c->d.U) return TBS_EINVAL;
    if (c->stream_cap == 0) return TBS_EINVAL;   // no stream_buffer_frames in the configuration
    c->h_T.assign(U, 0);
    std::vector<int32_t> off(U + 1, 0);
    c->s_fill.assign(U, 0);
    c->streaming = true;
    return begin_batch(c, c->stream_enc, off.data(), U, 0, 0);
}

static int segment_begin(tbs_ctx *c, int32_t seg_index, int32_t *rows_host);

int tbs_segment_begin(tbs_ctx *c, int32_t seg_index, int32_t *rows_host) {
    if (!c || seg_index < 0) return TBS_EINVAL;
    if (c->streaming) return TBS_ESTATE;   // a stream's segments are started by tbs_push_segment
    return segment_begin(c, seg_index, rows_host);
}

static int segment_begin(tbs_ctx *c, int32_t seg_index, int32_t *rows_host) {
    if (c->state != ST_BEGUN && c->state != ST_READY && c->state != ST_SELECTED) return TBS_ESTATE;
    if (c->state != ST_BEGUN && c->h_counts[TBS_CNT_PAIRS] != 0) return TBS_ESTATE;  // A not empty yet
    c->seg = seg_index;
    c->round = 0;
    c->pred_ahead = 0;
    c->join_ahead = false;
    AView &A = c->A[c->a_cur];
    HIPCHK(c, launch_segment_begin(c->stream, c->cur, c->seg, c->utt_T, c->B, A, c->rv, c->pool_p, c->pool_h,
                                   c->pool_c, c->pool_rows));
    HIPCHK(c, launch_rowfill(c->stream, c->cur, c->seg, c->utt_off, A, c->rv, c->nodes, 0, c->h_counts_dev, ++c->seq));
    // The joiner input rows of the first round go out before the counts are known, on the largest
    // grid a round can need (the kernel takes the row count from device memory): it runs while the
    // host waits for the counts and enqueues the GEMM.
    {
        const Dims &d = c->cur;
        ProfScope ps(c, TBS_K_PREP, 0);
        HIPCHK(c, joiner_rows(c, d.U * d.N * d.S, c->rv.counts + TBS_CNT_ROWS));
        c->prep_ahead = true;
    }
    HIPCHK(c, wait_counts(c));
    if (rows_host) *rows_host = c->h_counts[TBS_CNT_ROWS];
    c->state = ST_READY;
    return TBS_OK;
}

// A joiner call may be run in pieces of whole hypotheses: input rows, GEMM and expansion of one
// piece, then the next, so that the expansion reads the logits of a piece while they are still
// in the memory-side cache (256 MB on this part) instead of after the GEMM has pushed them out to
// memory.  Every piece's logits still go to their place in the full array, which
// tbs_select_merge reads a few values of.  Off unless the configuration asks for it: measured on
// the largest configuration (51200 rows x 4096, pieces of 12288 rows = 192 MB) the expansion
// launches do read faster (5.2 against 4.4 TB/s) but the GEMM loses more in its five shorter
// launches, and the whole decode ran 4 % slower (295 against 283 ms).
// Returns the rows of a piece, 0 for a call that is not split.
static int joiner_piece_rows(const tbs_ctx *c, int rows) {
    if (c->cfg.dtype != 1 || c->cfg.joiner_chunk_rows <= 0) return 0;
    return rows > c->cfg.joiner_chunk_rows ? c->cfg.joiner_chunk_rows : 0;
}

static int joiner_expand_pieces(tbs_ctx *c, int rows, int piece) {
    const Dims &d = c->cur;
    const int pairs = c->h_counts[TBS_CNT_PAIRS];
    const int P = std::max(1, piece / d.S);   // hypotheses per piece (each has at most S rows)
    int left = rows;
    for (int p0 = 0; p0 < pairs; p0 += P) {
        const int p1 = std::min(pairs, p0 + P), m_max = (p1 - p0) * d.S;
        // the piece's rows are those of its hypotheses: known on the device only (segments may be ragged)
        const int *rb = c->rv.pair_row0 + p0;
        const int *re = p1 < pairs ? c->rv.pair_row0 + p1 : c->rv.counts + TBS_CNT_ROWS;
        const int units = p1 == pairs ? left : std::min(m_max, left);
        left -= units;
        if (!c->prep_ahead) {
            ProfScope ps(c, TBS_K_PREP, units);
            HIPCHK(c, launch_joiner_prep(c->stream, d, c->cfg.dtype, c->cfg.act, m_max, c->enc, c->pool_p, c->rv, c->amat,
                                         re, rb));
        }
        {
            ProfScope ps(c, TBS_K_JOINER, units);
            ProfScope pg(c, TBS_K_GEMM, (int64_t)units * d.V * d.Dj);
            HIPCHK(c, launch_gemm_bf16_rows(c->stream, (const bf16_t *)c->amat, (const bf16_t *)c->w.w_out, c->w.b_out,
                                            c->logits, m_max, d.V, d.Dj, d.V, rb, re));
        }
        {
            ProfScope ps(c, TBS_K_EXPAND, units);
            HIPCHK(c, launch_expand(c->stream, d, p1 - p0, c->logits, c->A[c->a_cur], c->rv, c->row_lc, c->dphi,
                                    c->cand_score, c->cand_tok, c->row_stats, c->delta_nb, (c->cfg.debug & 2) != 0,
                                    nullptr, p0));
        }
    }
    c->prep_ahead = false;
    c->expanded_ahead = true;
    return TBS_OK;
}

int tbs_joiner_segment(tbs_ctx *c) {
    if (!c) return TBS_EINVAL;
    if (c->state != ST_READY) return TBS_ESTATE;
    const int rows = c->h_counts[TBS_CNT_ROWS];
    if (c->round + 1 > c->cur.R) return TBS_EOVERFLOW;
    c->round += 1;
    if (c->join_ahead) {   // enqueued behind the predictor step, before the counts were known
        c->join_ahead = false;
        c->prep_ahead = false;
        if (c->prof_kernel == TBS_K_JOINER) c->prof_units += rows;
        if (c->prof_kernel == TBS_K_GEMM) c->prof_units += (int64_t)rows * c->cur.V * c->cur.Dj;
        c->n_launches += 1;
        c->state = ST_JOINED;
        return TBS_OK;
    }
    if (const int piece = joiner_piece_rows(c, rows)) {
        const int rc = joiner_expand_pieces(c, rows, piece);
        if (rc) return rc;
        c->n_launches += 1;
        c->state = ST_JOINED;
        return TBS_OK;
    }
    if (!c->prep_ahead) {
        ProfScope ps(c, TBS_K_PREP, rows);
        HIPCHK(c, joiner_rows(c, rows, nullptr));
    }
    c->prep_ahead = false;
    {
        ProfScope ps(c, TBS_K_JOINER, rows);
        HIPCHK(c, gemm(c, c->amat, c->w.w_out, c->w.b_out, c->logits, rows, c->cur.V, c->cur.Dj, nullptr,
                       c->cur.V));
    }
    c->n_launches += 1;
    c->state = ST_JOINED;
    return TBS_OK;
}

int tbs_expand(tbs_ctx *c) {
    if (!c) return TBS_EINVAL;
    if (c->state != ST_JOINED) return TBS_ESTATE;
    if (c->expanded_ahead) {   // a large call: each piece was expanded right behind its GEMM
        c->expanded_ahead = false;
        c->state = ST_EXPANDED;
        return TBS_OK;
    }
    const int pairs = c->h_counts[TBS_CNT_PAIRS];
    {
        ProfScope ps(c, TBS_K_EXPAND, c->h_counts[TBS_CNT_ROWS]);
        HIPCHK(c, launch_expand(c->stream, c->cur, pairs, c->logits, c->A[c->a_cur], c->rv, c->row_lc, c->dphi,
                                c->cand_score, c->cand_tok, c->row_stats, c->delta_nb, (c->cfg.debug & 2) != 0));
    }
    c->state = ST_EXPANDED;
    return TBS_OK;
}

static int predictor_launch(tbs_ctx *c, int M, const int *m_dev, int part = 0, const int *any_dev = nullptr);

// Expansion and select/merge of a round in one kernel (small shapes, see round_kernels.hip)?  Not
// when the generic expansion kernel is forced, the fusion switched off (debug bit 7), the expansion
// already done piece by piece behind the joiner, or one of the two steps being timed on its own.
static bool round_fused_ok(const tbs_ctx *c) {
    return !(c->cfg.debug & (2 | 128)) && !c->expanded_ahead && c->prof_kernel != TBS_K_EXPAND &&
           c->prof_kernel != TBS_K_SELECT && round_fits(c->cur);
}

static int select_merge_impl(tbs_ctx *c, int32_t *live_host, bool fused);

int tbs_select_merge(tbs_ctx *c, int32_t *live_host) {
    if (!c) return TBS_EINVAL;
    if (c->state != ST_EXPANDED) return TBS_ESTATE;
    return select_merge_impl(c, live_host, false);
}

// fused: the state is "joined"; one kernel runs the expansion and select/merge
static int select_merge_impl(tbs_ctx *c, int32_t *live_host, bool fused) {
    AView &A = c->A[c->a_cur], &An = c->A[c->a_cur ^ 1];
    const int drop = c->cfg.max_rounds_per_segment > 0 && c->round >= c->cfg.max_rounds_per_segment;
    bool gathered = false;
    {
        ProfScope ps(c, fused ? TBS_K_ROUND : TBS_K_SELECT, c->h_counts[TBS_CNT_PAIRS]);
        if (fused)
            HIPCHK(c, launch_round(c->stream, c->cur, c->round, drop, c->logits, A, An, c->B, c->rv, c->nodes,
                                   c->row_stats, c->delta_nb));
        else
            HIPCHK(c, launch_select_merge(c->stream, c->cur, c->round, drop, c->logits, c->row_lc, c->dphi,
                                          c->cand_score, c->cand_tok, A, An, c->B, c->rv, c->nodes));
        // small batches: the row list kernel also writes the first LSTM layer's input rows
        const bool fused_gather = c->emb_gates && !(c->cfg.debug & 32) && (c->cur.H & 3) == 0 &&
                                  (long)c->cur.U * c->cur.N <= 1024;
        HIPCHK(c, launch_rowfill(c->stream, c->cur, c->seg, c->utt_off, An, c->rv, c->nodes, 1, c->h_counts_dev,
                                 ++c->seq, fused_gather ? c->pool_h : nullptr,
                                 fused_gather ? (bf16_t *)c->xh[0] : nullptr));
        gathered = fused_gather;
    }
    // Otherwise the first kernel of the predictor step goes out before the counts are known, on the
    // largest grid the round could need (it sizes itself from device memory): it runs while the host
    // waits for the counts and enqueues the rest, which would otherwise leave the GPU idle.
    if (!gathered) {
        ProfScope ps(c, TBS_K_PREDICTOR, 0);
        if (c->emb_gates)
            HIPCHK(c, launch_pred_gather_h(c->stream, c->cur, c->cur.U * c->cur.N, An, c->rv, c->pool_h,
                                           (bf16_t *)c->xh[0]));
        else
            HIPCHK(c, launch_pred_gather(c->stream, c->cur, c->cfg.dtype, c->cur.U * c->cur.N, An, c->rv, c->w.embed,
                                         c->pool_h, c->xh[0]));
    }
    // Small batches: the LSTM layers of the predictor step go out now, sized for every hypothesis
    // the round could have created and reading the number it did create from device memory.  The
    // host's round trip (counts into pinned memory, the host seeing them, a launch reaching the GPU:
    // 7-8 us during which the GPU had nothing to run) then lies beside these kernels instead of in
    // front of them; the projection and the next round follow from tbs_predictor_step on, in time.
    // A round that created nothing (the last of every segment) pays launches that leave at once,
    // which is why no more than this goes out early: measured, the layers alone beat layers +
    // projection and layers + projection + next joiner GEMM (23.5 / 24.2 / 24.7 ms per decode).
    c->pred_ahead = 0;
    c->join_ahead = false;
    c->a_cur ^= 1;   // (the new hypotheses are the current group from here on)
    if (!(c->cfg.debug & 64) && predictor_all_fused(c, c->cur.U * c->cur.N)) {
        ProfScope ps(c, TBS_K_PREDICTOR, 0);
        const int rc = predictor_launch(c, c->cur.U * c->cur.N, c->rv.counts + TBS_CNT_PAIRS, 1);
        if (rc) return rc;
        c->pred_ahead = 1;
    }
    HIPCHK(c, wait_counts(c));
    if (live_host) *live_host = c->h_counts[TBS_CNT_PAIRS];
    c->state = ST_SELECTED;
    return check_err_flags(c);
}

// UpdatePredictorOutput for the first M pairs (or, with m_dev, for as many as *m_dev says once the
// kernels run: then M is the upper bound the launches are sized for, and only the forms that can
// read their row count from device memory may be used: see predictor_all_fused).
static bool predictor_all_fused(const tbs_ctx *c, int M, int max_tiles) {
    const Dims &d = c->cur;
    if (c->cfg.dtype != 1 || !c->emb_gates || (c->cfg.debug & (8 | 16))) return false;
    for (int l = 0; l < d.L; ++l)
        if (!gemm_lstm_fits(M, d.H, l == 0 ? d.H : 2 * d.H, max_tiles)) return false;
    return gemm_join_fits(M, d.Dj, d.H, max_tiles);
}

static int64_t predictor_madds(const tbs_ctx *c, int64_t pairs) {   // multiply-adds of its GEMMs
    const Dims &d = c->cur;
    int64_t n = pairs * d.Dj * d.H;
    for (int l = 0; l < d.L; ++l) {
        const int in_dim = l == 0 ? d.E : d.H;
        n += pairs * 4 * d.H * ((l == 0 && c->emb_gates) ? d.H : in_dim + d.H);
    }
    return n;
}

static int predictor_launch(tbs_ctx *c, int M, const int *m_dev, int part, const int *any_dev) {   // part: 0 all, 1 the LSTM layers, 2 the projection
    const Dims &d = c->cur;
    AView &A = c->A[c->a_cur];
    // (the input rows of the first layer were gathered behind select/merge)
    for (int l = 0; l < d.L && part != 2; ++l) {
        int in_dim = l == 0 ? d.E : d.H;
        const int K = (l == 0 && c->emb_gates) ? d.H : in_dim + d.H;
        if (c->emb_gates && !(c->cfg.debug & 8) && gemm_lstm_fits(M, d.H, K, c->fixed ? GS_TILES_FIXED : GS_TILES)) {
            // small problem: the cell update runs in the epilogue of the gate GEMM
            const bool last = l + 1 == d.L;
            LstmEp ep;
            ep.pslot = c->rv.pair_pslot;
            ep.slot = c->rv.pair_slot;
            ep.tok = c->rv.pair_tok;
            ep.emb_gates = l == 0 ? c->emb_gates_perm : nullptr;
            ep.c_par = c->pool_c + (size_t)l * c->pool_rows * d.H;
            ep.c_new = c->pool_c + (size_t)l * c->pool_rows * d.H;
            ep.h_new = c->pool_h + (size_t)l * c->pool_rows * d.H;
            ep.h_par_next = last ? nullptr : c->pool_h + (size_t)(l + 1) * c->pool_rows * d.H;
            ep.out16 = (bf16_t *)(last ? c->htop : c->xh[(l + 1) & 1]);
            ep.H = d.H;
            ProfScope pg(c, TBS_K_GEMM, (m_dev || any_dev) ? 0 : (int64_t)M * 4 * d.H * K);
            HIPCHK(c, launch_gemm_lstm(c->stream, (const bf16_t *)c->xh[l & 1], (const bf16_t *)c->wperm[l], c->bperm[l],
                                       M, K, ep, m_dev, any_dev));
            continue;
        }
        if (m_dev || any_dev) return TBS_ESTATE;   // (predictor_all_fused was not asked)
        if (l == 0 && c->emb_gates)
            HIPCHK(c, gemm(c, c->xh[0], c->w.w_hh[0], nullptr, c->gates, M, 4 * d.H, d.H, nullptr, 4L * d.H));
        else
            HIPCHK(c, gemm(c, c->xh[l & 1], c->wcat[l], c->w.b_lstm[l], c->gates, M, 4 * d.H, in_dim + d.H, nullptr,
                           4L * d.H));
        HIPCHK(c, launch_lstm_pointwise(c->stream, d, c->cfg.dtype, M, l, A, c->rv, c->gates, c->pool_h, c->pool_c,
                                        c->pool_rows, c->xh[(l + 1) & 1], c->htop, l == 0 ? c->emb_gates : nullptr));
    }
    if (part == 1) return TBS_OK;
    if (c->cfg.dtype == 1 && !(c->cfg.debug & 16) && gemm_join_fits(M, d.Dj, d.H, c->fixed ? GS_TILES_FIXED : GS_TILES)) {
        // small problem: the projection's epilogue also makes the joiner input rows of the coming
        // round (every row of that round belongs to one of these pairs)
        JoinEp jp;
        jp.pair_row0 = c->rv.pair_row0;
        jp.pair_len = c->rv.pair_len;
        jp.pair_frame0 = c->rv.pair_frame0;
        jp.enc = (const bf16_t *)c->enc;
        jp.amat = (bf16_t *)c->amat;
        jp.act = c->cfg.act;
        // (a small problem leaves most CUs idle: as many workgroups per tile as the segment has frames,
        // each forming the joiner input rows of one frame, while they fit one wave of workgroups)
        {
            const long tiles = (long)((M + 63) / 64) * ((d.Dj + 63) / 64);
            jp.fgroups = (c->cfg.debug & 2048) ? 1 : (int)std::max(1L, std::min((long)d.S, 256 / std::max(tiles, 1L)));
        }
        ProfScope pg(c, TBS_K_GEMM, (m_dev || any_dev) ? 0 : (int64_t)M * d.Dj * d.H);
        HIPCHK(c, launch_gemm_join(c->stream, (const bf16_t *)c->htop, (const bf16_t *)c->w.w_proj, c->w.b_proj,
                                   c->pool_p, M, d.Dj, d.H, c->rv.pair_slot, d.Dj, jp, m_dev, any_dev));
        c->prep_ahead = true;
    } else {
        if (m_dev || any_dev) return TBS_ESTATE;
        HIPCHK(c, gemm(c, c->htop, c->w.w_proj, c->w.b_proj, c->pool_p, M, d.Dj, d.H, c->rv.pair_slot, d.Dj));
    }
    return TBS_OK;
}

int tbs_predictor_step(tbs_ctx *c) {
    if (!c) return TBS_EINVAL;
    if (c->state != ST_SELECTED) return TBS_ESTATE;
    const int pairs = c->h_counts[TBS_CNT_PAIRS];
    if (c->pred_ahead) {
        // the kernels went out behind select/merge, before the counts were known; now they are
        const int level = c->pred_ahead;
        c->pred_ahead = 0;
        c->prep_ahead = pairs > 0;   // (with no pairs the projection made no joiner input rows)
        // (work of the launches that went out with their size unknown; the projection, if it goes
        // out now, counts itself)
        if (c->prof_kernel == TBS_K_GEMM)
            c->prof_units += predictor_madds(c, pairs) - (level == 1 ? (int64_t)pairs * c->cur.Dj * c->cur.H : 0);
        if (c->prof_kernel == TBS_K_PREDICTOR) c->prof_units += pairs;
        if (level == 1 && pairs > 0) {
            ProfScope ps(c, TBS_K_PREDICTOR, 0);
            const int rc = predictor_launch(c, pairs, nullptr, 2);
            if (rc) return rc;
        }
    } else if (pairs > 0) {
        ProfScope ps(c, TBS_K_PREDICTOR, pairs);
        const int rc = predictor_launch(c, pairs, nullptr);
        if (rc) return rc;
    }
    c->state = ST_READY;
    return TBS_OK;
}

int tbs_result(tbs_ctx *c, int32_t *tokens, int32_t *lens, double *logscores, int32_t *nbest_count,
               int32_t max_len) {
    if (!c || !tokens || !lens || !logscores || !nbest_count || max_len < 1) return TBS_EINVAL;
    if (c->state == ST_INIT) return TBS_ESTATE;
    const Dims &d = c->cur;
    const long UN = (long)d.U * d.N;
    if (max_len > c->res_max_len) return TBS_EINVAL;   // the result buffer was sized at tbs_init (max_result_len)
    // (the kernel writes every entry of the four outputs: nothing is cleared beforehand)
    HIPCHK(c, launch_finalize(c->stream, d, c->B, c->nodes, c->res_count, c->res_len, c->res_logs, c->res_tok,
                              max_len));
    HIPCHK(c, hipMemcpyAsync(tokens, c->res_tok, sizeof(int) * UN * max_len, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(lens, c->res_len, sizeof(int) * UN, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(logscores, c->res_logs, sizeof(double) * UN, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(nbest_count, c->res_count, sizeof(int) * d.U, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    for (long i = 0; i < UN; ++i)
        if (lens[i] > max_len) return TBS_EOVERFLOW;   // truncated to max_len tokens; lens keeps the true length
    return TBS_OK;
}

// Small batches: the head of a segment and its whole first round enqueued in one go, with one
// wait at the end.  Every kernel that needs a count (rows for the joiner GEMM and its input rows,
// pairs for the expansion and the predictor step) reads it from device memory and is sized for
// the most the batch can have; the host's round trip after the first row list (7-8 us with
// nothing for the GPU to run) disappears.  Not while a kernel family is being timed (the brackets
// want the counts at launch).
static bool segment_ahead_ok(const tbs_ctx *c) {
    const Dims &d = c->cur;
    return !(c->cfg.debug & 64) && c->prof_kernel < 0 && c->cfg.dtype == 1 && d.R >= 1 &&
           gemm_small_fits(d.U * d.N * d.S, d.V, d.Dj) && predictor_all_fused(c, d.U * d.N);
}

static int segment_begin_ahead(tbs_ctx *c, int32_t seg_index) {
    if (c->state != ST_BEGUN && c->state != ST_READY && c->state != ST_SELECTED) return TBS_ESTATE;
    if (c->state != ST_BEGUN && c->h_counts[TBS_CNT_PAIRS] != 0) return TBS_ESTATE;  // A not empty yet
    const Dims &d = c->cur;
    c->seg = seg_index;
    c->round = 1;
    AView &A = c->A[c->a_cur], &An = c->A[c->a_cur ^ 1];
    const int *rows_dev = c->rv.counts + TBS_CNT_ROWS, *pairs_dev = c->rv.counts + TBS_CNT_PAIRS;
    // A = ChooseNBest(B), B = [], the row list, the joiner input rows
    HIPCHK(c, launch_segment_begin(c->stream, d, c->seg, c->utt_T, c->B, A, c->rv, c->pool_p, c->pool_h, c->pool_c,
                                   c->pool_rows));
    HIPCHK(c, launch_rowfill(c->stream, d, c->seg, c->utt_off, A, c->rv, c->nodes, 0, c->h_counts_dev, ++c->seq));
    HIPCHK(c, joiner_rows(c, d.U * d.N * d.S, rows_dev));
    // first round: joiner, expansion, select/merge, row list, predictor step
    HIPCHK(c, launch_gemm_bf16(c->stream, (const bf16_t *)c->amat, (const bf16_t *)c->w.w_out, c->w.b_out, c->logits,
                               d.U * d.N * d.S, d.V, d.Dj, nullptr, d.V, 0, rows_dev));
    c->n_launches += 1;
    const int drop = c->cfg.max_rounds_per_segment > 0 && c->round >= c->cfg.max_rounds_per_segment;
    if (round_fused_ok(c)) {
        HIPCHK(c, launch_round(c->stream, d, c->round, drop, c->logits, A, An, c->B, c->rv, c->nodes, c->row_stats,
                               c->delta_nb));
    } else {
        HIPCHK(c, launch_expand(c->stream, d, d.U * d.N, c->logits, A, c->rv, c->row_lc, c->dphi, c->cand_score,
                                c->cand_tok, c->row_stats, c->delta_nb, (c->cfg.debug & 2) != 0, pairs_dev));
        HIPCHK(c, launch_select_merge(c->stream, d, c->round, drop, c->logits, c->row_lc, c->dphi, c->cand_score,
                                      c->cand_tok, A, An, c->B, c->rv, c->nodes));
    }
    const bool fused_gather = !(c->cfg.debug & 32) && (d.H & 3) == 0 && (long)d.U * d.N <= 1024;
    HIPCHK(c, launch_rowfill(c->stream, d, c->seg, c->utt_off, An, c->rv, c->nodes, 1, c->h_counts_dev, ++c->seq,
                             fused_gather ? c->pool_h : nullptr, fused_gather ? (bf16_t *)c->xh[0] : nullptr));
    if (!fused_gather)
        HIPCHK(c, launch_pred_gather_h(c->stream, d, d.U * d.N, An, c->rv, c->pool_h, (bf16_t *)c->xh[0]));
    c->a_cur ^= 1;
    const int rc = predictor_launch(c, d.U * d.N, pairs_dev);
    if (rc) return rc;
    c->prep_ahead = false;
    c->pred_ahead = 2;
    c->join_ahead = false;
    if (c->round + 1 <= d.R) {   // and the joiner GEMM of the second round
        HIPCHK(c, launch_gemm_bf16(c->stream, (const bf16_t *)c->amat, (const bf16_t *)c->w.w_out, c->w.b_out, c->logits,
                                   d.U * d.N * d.S, d.V, d.Dj, nullptr, d.V, 0, rows_dev));
        c->join_ahead = true;
    }
    HIPCHK(c, wait_counts(c));
    c->state = ST_SELECTED;
    return check_err_flags(c);
}

// expansion and select/merge behind a joiner call: one kernel where the shape allows, else two
static int expand_select(tbs_ctx *c, int32_t *live) {
    if (c->state != ST_JOINED) return TBS_ESTATE;
    if (round_fused_ok(c)) return select_merge_impl(c, live, true);
    const int rc = tbs_expand(c);
    return rc ? rc : tbs_select_merge(c, live);
}

// Wait until every utterance's workgroup of launch `seq` has told the host its count (slot layout):
// one word per utterance in pinned memory, in the half that launch writes to.  The counts go to
// `out` [U].  Bounded like wait_counts.
static int wait_live(tbs_ctx *c, int seq, int *out, int *total, bool *trie_full) {
    const int U = c->cur.U;
    const unsigned want = (unsigned)seq & 0xFFFFFFu;
    const int *words = c->h_live + (seq & 1) * c->cur.U;
    std::chrono::steady_clock::time_point t0;
    bool timing = false;
    int u = 0, sum = 0;
    bool full = false;
    for (unsigned spin = 1; u < U; ++spin) {
        const int w = __atomic_load_n(&words[u], __ATOMIC_ACQUIRE);
        if (((unsigned)w >> 8) == want) {
            out[u] = w & 63;
            sum += w & 63;
            full = full || (w & 64);
            ++u;
            continue;
        }
        if ((spin & 0x3FFFFF) == 0) {
            const hipError_t e = hipStreamQuery(c->stream);
            if (e == hipSuccess) {
                if (((unsigned)__atomic_load_n(&words[u], __ATOMIC_ACQUIRE) >> 8) == want) continue;
                c->last_hip = (int)hipErrorUnknown;
                return TBS_EHIP;
            }
            if (e != hipErrorNotReady) {
                c->last_hip = (int)e;
                return TBS_EHIP;
            }
            const auto now = std::chrono::steady_clock::now();
            if (!timing) {
                t0 = now;
                timing = true;
            } else if (now - t0 > std::chrono::seconds(TBS_WAIT_LIMIT_S)) {
                c->last_hip = (int)hipErrorLaunchTimeOut;
                return TBS_EHIP;
            }
        }
    }
    *total = sum;
    *trie_full = full;
    return TBS_OK;
}

// One segment in the slot layout: four kernels a round (joiner GEMM; expansion, select/merge and
// the utterance's own bookkeeping; LSTM layers; projection), no row list kernel, and the host
// reads one word per utterance instead of waiting for a scan over all of them.  The head of the
// segment and its first round go out without a wait between them: every kernel finds what it
// needs to know of an utterance in that utterance's descriptors.
static int run_segment_fixed(tbs_ctx *c, int32_t seg_index) {
    if (c->state != ST_BEGUN && c->state != ST_READY && c->state != ST_SELECTED) return TBS_ESTATE;
    const Dims &d = c->cur;
    c->seg = seg_index;
    c->round = 0;
    c->live_u.assign(d.U, 0);
    FixedView fx{};
    fx.on = 1;
    fx.seg = seg_index;
    fx.utt_off = c->utt_off;
    fx.fig = c->utt_fig;
    fx.live_sum = c->live_sum;
    fx.host_live = c->h_live_dev;
    fx.pool_h = c->pool_h;
    fx.xh = (bf16_t *)c->xh[0];
    // A = ChooseNBest(B), B = [], the first round's pair descriptors and joiner input rows
    const int head_seq = fx.seq = ++c->seq;
    // (the head kernel also forms the first round's joiner input rows where it moves p in 16-byte pieces
    // and the segment's frames fit the LDS it keeps for them; a kernel of their own makes them otherwise,
    // or where debug bit 10 asks for it)
    const bool rows_in_head = ((d.Dj | d.H) & 3) == 0 && d.Dj <= 1024 && d.S <= TBS_FIXED_SMAX &&
                              !(c->cfg.debug & 1024);
    fx.amat = rows_in_head ? (bf16_t *)c->amat : nullptr;
    fx.enc = (const bf16_t *)c->enc;
    fx.act = c->cfg.act;
    fx.parts = d.U > 256 ? 1 : (d.U > 128 ? 2 : 4);   // (a small batch leaves most CUs idle: several workgroups share an utterance)
    HIPCHK(c, launch_segment_begin(c->stream, d, c->seg, c->utt_T, c->B, c->A[c->a_cur], c->rv, c->pool_p, c->pool_h,
                                   c->pool_c, c->pool_rows, &fx));
    if (!rows_in_head) {
        ProfScope ps(c, TBS_K_PREP, 0);
        HIPCHK(c, launch_joiner_prep_fixed(c->stream, d, c->cfg.act, (const bf16_t *)c->enc, c->pool_p, c->rv,
                                           (bf16_t *)c->amat));
    }
    fx.amat = nullptr;
    const int M = d.U * d.N * d.S;
    // (a row range per XCD in the joiner GEMM, the round kernel's workgroups on the XCD of their
    // utterance's rows, where every XCD gets rows, its range holds whole utterances and its tiles fit
    // its 32 CUs, two workgroups each)
    {
        const int rpx = gemm_small_xcd_rows(M);
        const long wgs = (long)(rpx / 64) * ((d.V + 63) / 64);
        const long tiles = (long)((M + 63) / 64) * ((d.V + 63) / 64);   // (more than 256: two workgroups share a CU)
        fx.xcd_rows = (!(c->cfg.debug & 4096) && (M + 63) / 64 >= 8 && d.N * d.S <= rpx && wgs <= (tiles > 256 ? 64 : 32)) ? rpx : 0;
    }
    // (S = 1 without logits: the GEMM's partials go out per 16-column piece where the round kernel's wave
    // has a lane for each of them, which spares the GEMM the merge of a tile's four)
    const int s1_pieces = (d.V + 63) / 64 <= 16 && !(c->cfg.debug & 16384) ? 1 : 0;
    std::vector<int> made(d.U, 0);
    int total = 0, rc;
    bool full = false, first = true;
    for (;;) {   // while Length(A) > 0
        if (c->round + 1 > d.R) return TBS_EOVERFLOW;
        c->round += 1;
        {
            ProfScope ps(c, TBS_K_JOINER, 0);
            ProfScope pg(c, TBS_K_GEMM, 0);
            if (c->s1) {
                const PartEp pe{c->part, d.N, d.blank, s1_pieces, fx.xcd_rows};
                HIPCHK(c, launch_gemm_part(c->stream, (const bf16_t *)c->amat, (const bf16_t *)c->w.w_out, c->w.b_out, M, d.V,
                                           d.Dj, pe));
            } else {
                HIPCHK(c, launch_gemm_bf16(c->stream, (const bf16_t *)c->amat, (const bf16_t *)c->w.w_out, c->w.b_out,
                                           c->logits, M, d.V, d.Dj, nullptr, d.V, 4, nullptr, fx.xcd_rows != 0));
            }
        }
        AView &A = c->A[c->a_cur], &An = c->A[c->a_cur ^ 1];
        const int drop = c->cfg.max_rounds_per_segment > 0 && c->round >= c->cfg.max_rounds_per_segment;
        fx.seq = ++c->seq;
        {
            ProfScope ps(c, TBS_K_ROUND, 0);
            if (c->s1) {
                HIPCHK(c, launch_round_s1(c->stream, d, c->round, drop, c->part, ((d.V + 63) / 64) * (s1_pieces ? 4 : 1), A, An, c->B, c->rv,
                                          c->nodes, &fx));
            } else {
                HIPCHK(c, launch_round(c->stream, d, c->round, drop, c->logits, A, An, c->B, c->rv, c->nodes,
                                       c->row_stats, c->delta_nb, &fx));
            }
        }
        c->a_cur ^= 1;
        // The LSTM layers go out before the host knows whether the round made anything (they leave at
        // once if it did not): the host's wait then lies beside them, not in front of them.
        const int *any = c->live_sum + (fx.seq & 1);
        {
            ProfScope ps(c, TBS_K_PREDICTOR, 0);
            if ((rc = predictor_launch(c, d.U * d.N, nullptr, 1, any))) return rc;
        }
        if ((rc = wait_live(c, fx.seq, made.data(), &total, &full))) return rc;
        // (the projection goes out the moment the host knows that the round made something: the LSTM
        // layers in front of it take about as long as seeing the words and making this call)
        if (!full && total > 0) {
            ProfScope ps(c, TBS_K_PREDICTOR, 0);
            if ((rc = predictor_launch(c, d.U * d.N, nullptr, 2, any))) return rc;
        }
        if (first) {   // (what the head of the segment put into A: there for certain once the round's words are)
            int t0 = 0;
            bool f0 = false;
            if ((rc = wait_live(c, head_seq, c->live_u.data(), &t0, &f0))) return rc;
            first = false;
        }
        // the joiner call that just ran: counted per utterance that had hypotheses in it
        int rows = 0, pairs = 0;
        for (int u = 0; u < d.U; ++u)
            if (c->live_u[u] > 0) {
                const int left = c->h_T[u] - seg_index * d.S, sp = left < 0 ? 0 : (left > d.S ? d.S : left);
                c->fx_calls += 1;
                c->fx_joined += sp;
                rows += c->live_u[u] * sp;
                pairs += c->live_u[u];
            }
        if (rows > 0) c->n_launches += 1;
        if (c->prof_kernel == TBS_K_JOINER) c->prof_units += rows;
        if (c->prof_kernel == TBS_K_GEMM) c->prof_units += (int64_t)rows * d.V * d.Dj + predictor_madds(c, total);
        if (c->prof_kernel == TBS_K_ROUND) c->prof_units += pairs;
        if (c->prof_kernel == TBS_K_PREDICTOR) c->prof_units += total;
        c->live_u = made;
        c->h_counts[TBS_CNT_PAIRS] = total;
        if (full) return TBS_EOVERFLOW;
        if (total == 0) break;
    }
    c->h_counts[TBS_CNT_ROWS] = 0;
    c->prep_ahead = false;
    c->state = ST_SELECTED;
    return TBS_OK;
}

// one segment: the head of the outer loop of Algorithm 1 and its inner loop (while Length(A) > 0)
static int run_segment(tbs_ctx *c, int32_t seg_index) {
    if (c->fixed) return run_segment_fixed(c, seg_index);
    int rc, rows = 0, live = 0;
    if (segment_ahead_ok(c)) {
        if ((rc = segment_begin_ahead(c, seg_index))) return rc;
    } else {
        if ((rc = segment_begin(c, seg_index, &rows))) return rc;
        if (rows == 0) return TBS_OK;
        if ((rc = tbs_joiner_segment(c))) return rc;
        if ((rc = expand_select(c, &live))) return rc;
    }
    for (;;) {
        if ((rc = tbs_predictor_step(c))) return rc;
        if (c->h_counts[TBS_CNT_ROWS] == 0) return TBS_OK;
        if ((rc = tbs_joiner_segment(c))) return rc;
        if ((rc = expand_select(c, &live))) return rc;
    }
}

int tbs_push_segment(tbs_ctx *c, const void *enc_proj, const int32_t *frame_offsets, int32_t flush) {
    if (!c || !frame_offsets) return TBS_EINVAL;
    if (!c->streaming || c->state == ST_INIT) return TBS_ESTATE;
    if (c->state != ST_BEGUN && c->h_counts[TBS_CNT_PAIRS] != 0) return TBS_ESTATE;   // a segment is under way
    const Dims &d = c->cur;
    const int U = d.U, S = d.S, cap = c->stream_cap;
    if (frame_offsets[0] != 0) return TBS_EINVAL;
    for (int u = 0; u < U; ++u) {
        const int n = frame_offsets[u + 1] - frame_offsets[u];
        if (n < 0 || c->s_fill[u] + n > cap) return TBS_EINVAL;
    }
    if (c->n_frames + frame_offsets[U] > c->cfg.max_frames_total) return TBS_EINVAL;
    if (frame_offsets[U] > 0 && !enc_proj) return TBS_EINVAL;
    HIPCHK(c, hipSetDevice(c->cfg.device_id));
    const long row_bytes = (long)d.Dj * elem_bytes(c);
    // Pinned descriptor areas, one per use within a call (the stream reads them later than the host
    // writes them); the call ends with the stream drained, so the next call may write them again.
    // The first area mirrors the device's: step sizes, first frames, then the descriptors of the copy that
    // appends the new frames, so that the first decode step of a push needs one copy for all three.
    const int Um = c->d.U;
    int *take = c->h_desc, *first = take + Um;                           // a decode step
    int *src = first + Um + 1, *dst = src + U, *cnt = src + 2 * U;       // appending the new frames
    int *src1 = c->h_desc + 5 * Um + 1, *dst1 = src1 + U, *cnt1 = src1 + 2 * U;   // leftovers to the spare area
    int *src2 = c->h_desc + 8 * Um + 1, *dst2 = src2 + U, *cnt2 = src2 + 2 * U;   // and back to the front
    const bool append = frame_offsets[U] > 0;
    if (append) {
        for (int u = 0; u < U; ++u) {
            src[u] = frame_offsets[u];
            dst[u] = u * cap + c->s_fill[u];
            cnt[u] = frame_offsets[u + 1] - frame_offsets[u];
            c->s_fill[u] += cnt[u];
        }
        c->n_frames += frame_offsets[U];
    }
    // decode: every utterance with a whole segment buffered (or, at a flush, with anything
    // buffered) takes one step; utterances advance independently of each other
    std::vector<int> pos(U, 0);
    for (int step = 0;; ++step) {
        bool any = false;
        for (int u = 0; u < U; ++u) {
            const int avail = c->s_fill[u] - pos[u];
            take[u] = avail >= S ? S : (flush ? avail : 0);
            first[u] = u * cap + pos[u];
            any = any || take[u] > 0;
        }
        if (step == 0 && append) {
            HIPCHK(c, hipMemcpyAsync(c->utt_T, take, sizeof(int) * (2 * (size_t)Um + 1 + 3 * (size_t)U), hipMemcpyHostToDevice,
                                     c->stream));
            HIPCHK(c, launch_stream_copy(c->stream, U, enc_proj, c->stream_enc, c->d_desc, row_bytes));
        } else if (any) {
            HIPCHK(c, hipMemcpyAsync(c->utt_T, take, sizeof(int) * (2 * (size_t)Um), hipMemcpyHostToDevice, c->stream));
        }
        if (!any) break;
        for (int u = 0; u < U; ++u) c->h_T[u] = take[u];   // (the slot layout's host bookkeeping reads the step sizes)
        const int rc = run_segment(c, 0);   // (waits for counts: the copy above is done by then)
        if (rc) return rc;
        for (int u = 0; u < U; ++u) pos[u] += take[u];
    }
    // what is left (less than a segment) moves to the front of its buffer, through the spare area
    bool left = false;
    for (int u = 0; u < U; ++u) {
        const int n = c->s_fill[u] - pos[u];
        src1[u] = u * cap + pos[u];
        dst1[u] = src2[u] = u * S;
        dst2[u] = u * cap;
        cnt1[u] = cnt2[u] = pos[u] > 0 ? n : 0;
        left = left || cnt1[u] > 0;
        c->s_fill[u] = n;
    }
    if (left) {
        HIPCHK(c, hipMemcpyAsync(c->d_desc, src1, sizeof(int) * 3 * U, hipMemcpyHostToDevice, c->stream));
        HIPCHK(c, launch_stream_copy(c->stream, U, c->stream_enc, c->stream_tmp, c->d_desc, row_bytes));
        HIPCHK(c, hipMemcpyAsync(c->d_desc, src2, sizeof(int) * 3 * U, hipMemcpyHostToDevice, c->stream));
        HIPCHK(c, launch_stream_copy(c->stream, U, c->stream_tmp, c->stream_enc, c->d_desc, row_bytes));
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return check_err_flags(c);
}

int tbs_decode(tbs_ctx *c, const void *enc_proj, const int32_t *frame_offsets, int32_t U, int32_t *tokens,
               int32_t *lens, double *logscores, int32_t *nbest_count, int32_t max_len) {
    int rc = tbs_begin(c, enc_proj, frame_offsets, U);
    if (rc) return rc;
    const int S = c->cur.S;
    const int nseg = (c->max_T + S - 1) / S;
    for (int seg = 0; seg < nseg; ++seg) {          // while t <= Length(enc)
        if ((rc = run_segment(c, seg))) return rc;
    }
    return tbs_result(c, tokens, lens, logscores, nbest_count, max_len);
}

int tbs_stats(const tbs_ctx *c, int64_t *joiner_calls, int64_t *joined_frames, int64_t *frames, int64_t *launches) {
    if (!c) return TBS_EINVAL;
    // (running sums kept by the row list kernel, as of the last counts the host waited for)
    if (joiner_calls) *joiner_calls = c->fixed ? c->fx_calls : c->h_counts[TBS_CNT_ACC_CALLS];
    if (joined_frames) *joined_frames = c->fixed ? c->fx_joined : c->h_counts[TBS_CNT_ACC_JOINED];
    if (frames) *frames = c->n_frames;
    if (launches) *launches = c->n_launches;
    return TBS_OK;
}

int tbs_path(const tbs_ctx *c) {
    if (!c) return TBS_EINVAL;
    if (c->state == ST_INIT) return TBS_ESTATE;
    return (c->fixed ? 1 : 0) | (c->s1 ? 2 : 0);
}

// ------------------------------------------------------------------ inspection
int tbs_debug_read(tbs_ctx *c, int32_t which, void *dst, size_t bytes) {
    if (!c || !dst) return TBS_EINVAL;
    if (c->state == ST_INIT) return TBS_ESTATE;
    const Dims &d = c->cur;
    const long UN = (long)d.U * d.N;
    const long pairs = c->h_counts[TBS_CNT_PAIRS], rows = c->h_counts[TBS_CNT_ROWS];
    const AView &A = c->A[c->a_cur];
    const void *src = nullptr;
    size_t have = 0;
    float *tmp = nullptr;
    switch (which) {
        case TBS_BUF_A_COUNT: src = A.count; have = sizeof(int) * d.U; break;
        case TBS_BUF_A_LOGS: src = A.logs; have = sizeof(double) * UN; break;
        case TBS_BUF_A_DHAT: src = A.dhat; have = sizeof(float) * UN * d.S; break;
        case TBS_BUF_A_PRED: {
            HIPCHK(c, hipMalloc((void **)&tmp, sizeof(float) * UN * d.Dj));
            HIPCHK(c, hipMemsetAsync(tmp, 0, sizeof(float) * UN * d.Dj, c->stream));
            HIPCHK(c, launch_gather_pred(c->stream, d, A, c->pool_p, tmp, 0));
            src = tmp;
            have = sizeof(float) * UN * d.Dj;
            break;
        }
        case TBS_BUF_LOGITS: src = c->logits; have = sizeof(float) * rows * d.V; break;
        case TBS_BUF_ROW_STATS:
            if (!c->row_stats) return TBS_ESTATE;
            src = c->row_stats; have = sizeof(float) * rows * 3; break;
        case TBS_BUF_DELTA_BLANK: src = c->dphi; have = sizeof(float) * pairs; break;
        case TBS_BUF_DELTA_NB:
            if (!c->delta_nb) return TBS_ESTATE;
            src = c->delta_nb; have = sizeof(float) * pairs * d.V; break;
        case TBS_BUF_CAND_SCORE: src = c->cand_score; have = sizeof(float) * pairs * d.N; break;
        case TBS_BUF_CAND_TOKEN: src = c->cand_tok; have = sizeof(int) * pairs * d.N; break;
        case TBS_BUF_PAIR_UTT: src = c->rv.pair_u; have = sizeof(int) * pairs; break;
        case TBS_BUF_PAIR_HYP: src = c->rv.pair_h; have = sizeof(int) * pairs; break;
        case TBS_BUF_PAIR_ROW0: src = c->rv.pair_row0; have = sizeof(int) * pairs; break;
        case TBS_BUF_PAIR_LEN: src = c->rv.pair_len; have = sizeof(int) * pairs; break;
        case TBS_BUF_COUNTS: src = c->rv.counts; have = sizeof(int) * 4; break;
        default: return TBS_EINVAL;
    }
    size_t n = std::min(have, bytes);
    hipError_t e = hipSuccess;
    if (n) e = hipMemcpyAsync(dst, src, n, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (tmp) (void)hipFree(tmp);
    HIPCHK(c, e);
    if (which == TBS_BUF_A_DHAT) {   // kept as logarithms, handed out as plain values
        float *v = (float *)dst;
        for (size_t i = 0; i < n / sizeof(float); ++i) v[i] = expf(v[i]);
    }
    return TBS_OK;
}

int tbs_debug_write(tbs_ctx *c, int32_t which, const void *src, size_t bytes) {
    if (c) c->prep_ahead = false;   // the state the rows were made from is being replaced
    if (!c || !src) return TBS_EINVAL;
    if (c->state == ST_INIT) return TBS_ESTATE;
    const Dims &d = c->cur;
    const long UN = (long)d.U * d.N;
    AView &A = c->A[c->a_cur];
    switch (which) {
        case TBS_BUF_A_COUNT:
            if (bytes != sizeof(int) * d.U) return TBS_EINVAL;
            HIPCHK(c, hipMemcpyAsync(A.count, src, bytes, hipMemcpyHostToDevice, c->stream));
            HIPCHK(c, launch_debug_fill_a(c->stream, d, A));
            break;
        case TBS_BUF_A_LOGS:
            if (bytes != sizeof(double) * UN) return TBS_EINVAL;
            HIPCHK(c, hipMemcpyAsync(A.logs, src, bytes, hipMemcpyHostToDevice, c->stream));
            break;
        case TBS_BUF_A_DHAT: {   // the library keeps logarithms; the caller gives and gets plain values
            if (bytes != sizeof(float) * UN * d.S) return TBS_EINVAL;
            std::vector<float> lg((size_t)UN * d.S);
            const float *v = (const float *)src;
            for (size_t i = 0; i < lg.size(); ++i) lg[i] = v[i] > 0.f ? logf(v[i]) : -INFINITY;
            HIPCHK(c, hipMemcpy(A.dhat, lg.data(), bytes, hipMemcpyHostToDevice));
            break;
        }
        case TBS_BUF_A_PRED: {
            if (bytes != sizeof(float) * UN * d.Dj) return TBS_EINVAL;
            float *tmp = nullptr;
            HIPCHK(c, hipMalloc((void **)&tmp, bytes));
            hipError_t e = hipMemcpyAsync(tmp, src, bytes, hipMemcpyHostToDevice, c->stream);
            if (e == hipSuccess) e = launch_gather_pred(c->stream, d, A, c->pool_p, tmp, 1);
            if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
            (void)hipFree(tmp);
            HIPCHK(c, e);
            break;
        }
        default: return TBS_EINVAL;
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return TBS_OK;
}

int tbs_debug_rebuild(tbs_ctx *c, int32_t seg_index, int32_t *rows_host) {
    if (!c || seg_index < 0) return TBS_EINVAL;
    if (c->state == ST_INIT) return TBS_ESTATE;
    c->seg = seg_index;
    c->round = 0;
    c->prep_ahead = false;
    HIPCHK(c, launch_set_sp(c->stream, c->cur, seg_index, c->utt_T, c->rv));
    HIPCHK(c, launch_rowfill(c->stream, c->cur, c->seg, c->utt_off, c->A[c->a_cur], c->rv, c->nodes, 0, c->h_counts_dev,
                             ++c->seq));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (rows_host) *rows_host = c->h_counts[TBS_CNT_ROWS];
    c->state = ST_READY;
    return TBS_OK;
}

int tbs_debug_hyps(tbs_ctx *c, int32_t group, int32_t *tokens, int32_t *lens, double *logscores, int32_t *counts,
                   int32_t cap, int32_t max_len) {
    if (!c || !tokens || !lens || !logscores || !counts || cap < 1 || max_len < 1 || group < 0 || group > 1)
        return TBS_EINVAL;
    if (c->state == ST_INIT) return TBS_ESTATE;
    const Dims &d = c->cur;
    const size_t n = (size_t)d.U * cap;
    int *dtok = nullptr, *dlen = nullptr, *dcnt = nullptr;
    double *dlogs = nullptr;
    hipError_t e = hipMalloc((void **)&dtok, sizeof(int) * n * max_len);
    if (e == hipSuccess) e = hipMalloc((void **)&dlen, sizeof(int) * n);
    if (e == hipSuccess) e = hipMalloc((void **)&dlogs, sizeof(double) * n);
    if (e == hipSuccess) e = hipMalloc((void **)&dcnt, sizeof(int) * d.U);
    if (e == hipSuccess)   // (the kernel writes every entry: nothing is cleared beforehand)
        e = launch_hyps_dump(c->stream, d, group, c->A[c->a_cur], c->B, c->nodes, cap, max_len, dtok, dlen, dlogs,
                             dcnt);
    if (e == hipSuccess) e = hipMemcpyAsync(tokens, dtok, sizeof(int) * n * max_len, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(lens, dlen, sizeof(int) * n, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(logscores, dlogs, sizeof(double) * n, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(counts, dcnt, sizeof(int) * d.U, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    (void)hipFree(dtok);
    (void)hipFree(dlen);
    (void)hipFree(dlogs);
    (void)hipFree(dcnt);
    HIPCHK(c, e);
    return TBS_OK;
}

int tbs_debug_hyps_noalloc(tbs_ctx *c, int32_t group, int32_t *tokens, int32_t *lens, double *logscores,
                           int32_t *counts, int32_t cap, int32_t max_len) {
    if (!c || !tokens || !lens || !logscores || !counts || cap < 1 || max_len < 1 || group < 0 || group > 1)
        return TBS_EINVAL;
    if (c->state == ST_INIT) return TBS_ESTATE;
    const Dims &d = c->cur;
    // layout inside the scratch: scores (8-byte entries first), tokens, lengths, counts
    const size_t n = (size_t)d.U * cap;
    const size_t b_logs = sizeof(double) * n, b_tok = sizeof(int) * n * (size_t)max_len, b_len = sizeof(int) * n,
                 b_cnt = sizeof(int) * (size_t)d.U;
    if ((size_t)cap > TBS_NOALLOC_BYTES || (size_t)max_len > TBS_NOALLOC_BYTES ||
        b_logs + b_tok + b_len + b_cnt > TBS_NOALLOC_BYTES)
        return TBS_ELIMIT;
    HIPCHK(c, hipSetDevice(c->cfg.device_id));
    unsigned char *base = (unsigned char *)g_scratch_ptr[c->cfg.device_id];   // resolved in tbs_init on this device
    if (!base) return TBS_ESTATE;
    double *dlogs = (double *)base;
    int *dtok = (int *)(base + b_logs), *dlen = (int *)(base + b_logs + b_tok),
        *dcnt = (int *)(base + b_logs + b_tok + b_len);
    // the kernel writes every entry of the four arrays, so what an earlier call left there does not matter
    HIPCHK(c, launch_hyps_dump(c->stream, d, group, c->A[c->a_cur], c->B, c->nodes, cap, max_len, dtok, dlen, dlogs,
                               dcnt));
    HIPCHK(c, hipMemcpyAsync(tokens, dtok, b_tok, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(lens, dlen, b_len, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(logscores, dlogs, b_logs, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(counts, dcnt, b_cnt, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return TBS_OK;
}

// ------------------------------------------------------------------ profiling
int tbs_profile_select(tbs_ctx *c, int32_t kernel_id) {
    if (!c || kernel_id < -1 || kernel_id >= TBS_K_COUNT) return TBS_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (kernel_id >= 0 && c->events.empty()) {
        c->events.resize(8192);
        for (auto &e : c->events) {
            HIPCHK(c, hipEventCreate(&e.a));
            HIPCHK(c, hipEventCreate(&e.b));
        }
    }
    c->prof_kernel = kernel_id;
    c->ev_used = 0;
    c->prof_units = 0;
    return TBS_OK;
}

int tbs_profile_read(tbs_ctx *c, int64_t *launches, double *total_ms, int64_t *units) {
    if (!c) return TBS_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    double tot = 0.0;
    for (size_t i = 0; i < c->ev_used; ++i) {
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, c->events[i].a, c->events[i].b));
        tot += ms;
    }
    if (launches) *launches = (int64_t)c->ev_used;
    if (total_ms) *total_ms = tot;
    if (units) *units = c->prof_units;
    c->ev_used = 0;
    c->prof_units = 0;
    return TBS_OK;
}

int tbs_profile_overhead(tbs_ctx *c, int32_t n, double *avg_us) {
    if (!c || n < 1 || !avg_us) return TBS_EINVAL;
    if (c->events.empty()) return TBS_ESTATE;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    double tot = 0.0;
    int done = 0;
    while (done < n) {
        const int batch = std::min<int>(n - done, (int)c->events.size());
        for (int i = 0; i < batch; ++i) {
            HIPCHK(c, hipEventRecord(c->events[i].a, c->stream));
            HIPCHK(c, launch_empty(c->stream));
            HIPCHK(c, hipEventRecord(c->events[i].b, c->stream));
        }
        HIPCHK(c, hipStreamSynchronize(c->stream));
        for (int i = 0; i < batch; ++i) {
            float ms = 0.f;
            HIPCHK(c, hipEventElapsedTime(&ms, c->events[i].a, c->events[i].b));
            tot += ms;
        }
        done += batch;
    }
    *avg_us = tot * 1e3 / n;
    return TBS_OK;
}

int tbs_gemm_bf16(const void *A, const void *B, const float *bias, float *C, int32_t M, int32_t N, int32_t K,
                  int32_t kernel, void *stream) {
    if (!A || !B || !C || M < 1 || N < 1 || K < 8 || K % 8 || kernel < 0 || kernel > 4) return TBS_EINVAL;
    if (kernel == 4 && K % 128) return TBS_EINVAL;
    hipError_t e = launch_gemm_bf16((hipStream_t)stream, (const bf16_t *)A, (const bf16_t *)B, bias, C, M, N, K,
                                    nullptr, N, kernel);
    return e == hipSuccess ? TBS_OK : TBS_EHIP;
}

}  // extern "C"
