// Second half of the inner loop of Algorithm 1 for one utterance, by one 64-lane wave: AddAndMerge of
// the blank expansions into B, ChooseNthScore, the joint ChooseNBestExpansions with the threshold
// test, and the new list A with its frame distributions.  Shared by the kernel that does this for
// every utterance of a batch and the kernel that runs a whole round of one utterance.
#pragma once
#include "tbs_internal.h"

#define WAVE 64

// log(exp(a) + exp(b)); the correction term lies in [0, log 2] and is taken in fp32
// (absolute error ~1e-7, far inside the score tolerance), the sum stays fp64
__device__ __forceinline__ double log_add(double a, double b) {
    double mx = a > b ? a : b, mn = a > b ? b : a;
    if (isinf(mx)) return mx;
    return mx + (double)log1pf(expf((float)(mn - mx)));
}

__device__ __forceinline__ u64 hash_append(u64 h, int token) {
    return (h ^ (u64)(unsigned)(token + 1)) * 0x100000001B3ull + 0x9E3779B97F4A7C15ull;
}

__device__ bool same_sequence(const int2 *nodes, int a, int b) {
    // both sequences have the same length, so the walks reach the root together
    while (a != b) {
        int2 na = nodes[a], nb = nodes[b];
        if (na.y != nb.y) return false;
        a = na.x;
        b = nb.x;
    }
    return true;
}

// The wave that runs select_merge_utt exchanges data between its lanes through LDS: the writes of
// all lanes are made visible before any lane reads (a single wave needs no barrier instruction).
__device__ __forceinline__ void sel_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

#define CAND_MAX (TBS_MAX_BEAM * TBS_MAX_BEAM)

// Figures for the host go out as uncached system-scope stores into pinned host memory, which the
// host polls while the stream runs on.
__device__ __forceinline__ void store_host(int *p, int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// What select_merge_utt leaves in LDS about the list A it made, for a caller that goes on with it.
struct SelectOut {
    int total;
    int nB;   // entries of B after the merge
    int slot[TBS_MAX_BEAM], pslot[TBS_MAX_BEAM], tok[TBS_MAX_BEAM], pnode[TBS_MAX_BEAM];
    int parent[TBS_MAX_BEAM];   // index in A of the hypothesis each new one was made from
};

// slot layout: descriptor of a pair that does not exist (every address made from it stays valid)
__device__ __forceinline__ void pair_mark_dead(const RowView &rv, int j, int u, int S) {
    rv.pair_u[j] = u;
    rv.pair_h[j] = 0;
    rv.pair_row0[j] = j * S;
    rv.pair_len[j] = 0;
    rv.pair_slot[j] = -1;
    rv.pair_pslot[j] = 0;
    rv.pair_frame0[j] = 0;
    rv.pair_tok[j] = 0;
}

// What the expansion step left for this utterance: logarithms and tokens of the N best expansions
// of each of its hypotheses [H, N], the logarithm of each blank expansion [H], and per frame of each
// hypothesis log(alpha_t / Z_t) - m_t [H, S'] (any of them in LDS or in device memory).
// Ranks by counting: the rank of entry i of v[0..n) is the number of entries that beat it (larger
// value, or equal value and earlier place; NaN beats nothing).  Every entry is read from LDS by all
// lanes that need it.  Up to 32 entries the wave's lanes share an entry's count (two lanes each up to
// 32, four up to 16), each counting over a part of the list, and add their counts up.
// fn(i, rank, value) is called once per entry, by one lane.
template <class F>
__device__ __forceinline__ void sel_rank(const double *v, int n, int lane, F fn) {
    if (n <= 32) {
        const int parts = n <= 16 ? 4 : 2, width = WAVE / parts;   // lanes per part
        const int i = lane & (width - 1), part = lane / width;
        const int per = (n + parts - 1) / parts, j0 = part * per, j1 = min(j0 + per, n);
        const double mine = v[min(i, n - 1)];
        int rank = 0;
#pragma unroll 4
        for (int j = j0; j < j1; ++j) {
            const double o = v[j];
            rank += (o > mine) || (o == mine && j < i);
        }
        rank += __shfl_xor(rank, 32);
        if (parts == 4) rank += __shfl_xor(rank, 16);
        if (part == 0 && i < n) fn(i, rank, mine);
    } else {
        for (int i = lane; i < n; i += WAVE) {
            const double mine = v[i];
            int rank = 0;
#pragma unroll 4
            for (int j = 0; j < n; ++j) {
                const double o = v[j];
                rank += (o > mine) || (o == mine && j < i);
            }
            fn(i, rank, mine);
        }
    }
}

#define SEL_PRE_FRAMES 8   // segments up to this long have their candidates' logits asked for ahead of the ranking

struct SelectIn {
    const float *cand_score;
    const int *cand_tok;
    const float *dphi;
    const float *lc;
    int slot_rows;   // 1: hypothesis h of the utterance owns the joiner rows h*S .. (slot layout); 0: rows h*S' ..
};

// What describes the utterance at the start of the step, in one round of loads.
struct SelectFigs {
    int sp, cntA, urow0, nB0, parity;
};
__device__ __forceinline__ SelectFigs select_figs(int u, const AView &A, const BView &B, const RowView &rv) {
    SelectFigs f;
    f.sp = rv.utt_sp[u];
    f.cntA = A.count[u];
    f.urow0 = rv.utt_row0[u];
    f.nB0 = B.count[u];
    f.parity = rv.utt_par[u];
    return f;
}

// s_dyn: LDS for the utterance's B list, BCAP * (8 + 8 + 3 * 4) bytes, 16-byte aligned.
// phase 0: the whole step.  phase 1: only what does not depend on the expansion (B and A staged in
// LDS); phase 2: the rest, by the same wave: a caller whose expansion runs in the same kernel does
// phase 1 beside it.  Phases 3, 4 and 5 are the parts of phase 2 (see below), for a caller that has two
// waves for them; the wave of phase 5 is the one that did phase 1 and 4 (`out->nB` is its).  (The phase is
// an argument, not a template parameter: the LDS arrays below belong to the function, and each
// instantiation of a template would have a set of its own.)
__device__ __forceinline__ void select_merge_utt(const int PHASE, const Dims &d, int round, int drop, int u, int lane,
                                                 const float *logits, SelectIn in, const SelectFigs &fg, AView A,
                                                 AView An, BView B, RowView rv, const int2 *nodes,
                                                 unsigned char *s_dyn, SelectOut *out = nullptr) {
    double *s_blogs = reinterpret_cast<double *>(s_dyn);
    u64 *s_bhash = reinterpret_cast<u64 *>(s_blogs + d.BCAP);
    int *s_bnode = reinterpret_cast<int *>(s_bhash + d.BCAP);
    int *s_blen = s_bnode + d.BCAP;
    int *s_bslot = s_blen + d.BCAP;
    __shared__ double s_key[CAND_MAX];
    __shared__ int s_ctok[CAND_MAX];
    __shared__ double s_alogs[TBS_MAX_BEAM];
    __shared__ u64 s_ahash[TBS_MAX_BEAM];
    __shared__ int s_anode[TBS_MAX_BEAM], s_alen[TBS_MAX_BEAM], s_aslot[TBS_MAX_BEAM];
    __shared__ double s_bkey[TBS_MAX_BEAM];
    __shared__ int s_match[TBS_MAX_BEAM];
    __shared__ int s_sel[TBS_MAX_BEAM];      // candidate index by rank
    __shared__ double s_thr;
    __shared__ int s_have_thr;
    __shared__ float s_dnew[TBS_MAX_SEG * TBS_MAX_BEAM];   // frame distributions of the new hypotheses, [frame][hypothesis]
    __shared__ float s_xpre[SEL_PRE_FRAMES * WAVE];        // logits of the candidates' tokens, [frame][candidate]
    const int N = d.N;
    const int sp = fg.sp, cntA = fg.cntA, urow0 = fg.urow0, nB0 = fg.nB0, parity = fg.parity;
    const int H = sp > 0 ? cntA : 0;
    if (H == 0) {
        if (lane == 0 && (PHASE == 0 || PHASE == 2 || PHASE == 5)) {
            An.count[u] = 0;
            if (out) out->total = 0;
        }
    } else {
        const long bbase = (long)u * d.BCAP;
        int nB = nB0;
        // --- stage B and A
        if (PHASE == 0 || PHASE == 1) {
            for (int i = lane; i < nB0; i += WAVE) {
                s_blogs[i] = B.logs[bbase + i];
                s_bhash[i] = B.hash[bbase + i];
                s_bnode[i] = B.node[bbase + i];
                s_blen[i] = B.len[bbase + i];
                s_bslot[i] = B.slot[bbase + i];
            }
            if (lane < H) {
                const long a = (long)u * N + lane;
                s_alogs[lane] = A.logs[a];
                s_ahash[lane] = A.hash[a];
                s_anode[lane] = A.node[a];
                s_alen[lane] = A.len[a];
                s_aslot[lane] = A.slot[a];
            }
            if (lane < N) s_sel[lane] = -1;
        }
        if (PHASE == 1) return;
        // The rest falls into three parts.  "Candidates" (keys of the per-hypothesis candidates, their
        // joint ranking, the logits of their tokens) and "merge" (AddAndMerge, the threshold) need
        // nothing of each other; "finish" needs both.  phase 0 and 2: one wave does all three; phase 3:
        // candidates only, phase 4: merge only, phase 5: finish only: a caller with a second wave to
        // spare runs 3 and 4 side by side and 5 behind a barrier.
        const bool do_cand = PHASE == 0 || PHASE == 2 || PHASE == 3;
        const bool do_merge = PHASE == 0 || PHASE == 2 || PHASE == 4;
        const bool do_finish = PHASE == 0 || PHASE == 2 || PHASE == 5;
        if (PHASE == 0) sel_sync();   // (A's scores, staged just above, are read by other lanes below)
        const int nc = H * N;
        const float rcp_n = __builtin_amdgcn_rcpf((float)N);   // c / N as (c + 0.5) * (1 / N): exact for c < 1024
        const bool pre_x = logits != nullptr && nc <= WAVE && sp <= SEL_PRE_FRAMES && !drop;
        float xpre[SEL_PRE_FRAMES];
        if (do_cand) {
            int tok_mine = -1;   // (token of candidate `lane`)
            for (int c = lane; c < nc; c += WAVE) {
                const int tok = in.cand_tok[c];
                if (c == lane) tok_mine = tok;
                s_ctok[c] = tok;
                s_key[c] = tok >= 0 ? s_alogs[(int)(((float)c + 0.5f) * rcp_n)] + (double)in.cand_score[c] : nan("");
            }
            // The d of a new hypothesis (below) needs the logits of its token at the S' frames.  Which
            // candidates become hypotheses is known only after the ranking, so where a lane per candidate
            // suffices the logits of every candidate's token are asked for now and wait in registers: their
            // round trip runs beside the merge and the ranking instead of behind them.
            if (pre_x) {
                const int c = min(lane, nc - 1), tokc = max(tok_mine, 0);
                const float *lrow = logits + (long)(urow0 + (int)(((float)c + 0.5f) * rcp_n) * (in.slot_rows ? d.S : sp)) * d.V + tokc;
#pragma unroll
                for (int q = 0; q < SEL_PRE_FRAMES; ++q) xpre[q] = lrow[(long)min(q, sp - 1) * d.V];
            }
        }
        if (do_merge) {
            // (dphi holds log delta_blank)
            if (lane < H) s_bkey[lane] = s_alogs[lane] + (double)in.dphi[lane];
            // --- AddAndMerge of every blank expansion.  The hypotheses of A are distinct sequences and so
            // are the entries of B, so each hypothesis matches at most one old entry and no entry added in
            // this round: all (hypothesis, entry) pairs are tested at once, matched scores are summed in
            // place, and the unmatched hypotheses are appended in hypothesis order.
            if (lane < H) s_match[lane] = -1;
            sel_sync();
            const float rcp_b = __builtin_amdgcn_rcpf((float)max(nB0, 1));   // (exact quotients up to 32 x 2048 pairs)
            for (int c = lane; c < H * nB0; c += WAVE) {
                const int h = (int)(((float)c + 0.5f) * rcp_b), i = c - h * nB0;
                if (s_bhash[i] == s_ahash[h] && s_blen[i] == s_alen[h] && same_sequence(nodes, s_bnode[i], s_anode[h]))
                    s_match[h] = i;
            }
            sel_sync();
            {
                const bool unmatched = lane < H && s_match[lane] < 0;
                const u64 um = __ballot(unmatched);
                const int n_new = __popcll(um);
                if (lane < H) {
                    if (!unmatched) {
                        const int f = s_match[lane];
                        s_blogs[f] = log_add(s_blogs[f], s_bkey[lane]);
                    } else {
                        const int pos = nB0 + __popcll(um & ((1ull << lane) - 1ull));
                        if (pos < d.BCAP) {
                            s_blogs[pos] = s_bkey[lane];
                            s_bhash[pos] = s_ahash[lane];
                            s_bnode[pos] = s_anode[lane];
                            s_blen[pos] = s_alen[lane];
                            s_bslot[pos] = s_aslot[lane];
                        } else {
                            atomicOr(&rv.counts[TBS_CNT_ERR], TBS_ERRF_BCAP);
                        }
                    }
                }
                nB = min(nB0 + n_new, d.BCAP);
            }
            sel_sync();
            // --- B back to memory: merged scores of old entries, and the new entries
            for (int i = lane; i < nB; i += WAVE) {
                B.logs[bbase + i] = s_blogs[i];
                if (i >= nB0) {
                    B.hash[bbase + i] = s_bhash[i];
                    B.node[bbase + i] = s_bnode[i];
                    B.len[bbase + i] = s_blen[i];
                    B.slot[bbase + i] = s_bslot[i];
                }
            }
            if (lane == 0) {
                B.count[u] = nB;
                if (out) out->nB = nB;
            }

            // --- threshold = ChooseNthScore(B, N), only defined when B holds N entries.  The rank of an
            // entry is the number of entries that beat it (larger score, or equal score and earlier
            // place); every lane counts for its own entries against the whole list, read from LDS at
            // one address for all lanes.  (Ranking by one ballot per entry was measured at ~270 ns per
            // entry on the single wave: readlane and ballot results are needed at once, so nothing
            // overlaps.)
            const bool have_thr_m = nB >= N;
            if (lane == 0) s_have_thr = have_thr_m;
            if (have_thr_m) sel_rank(s_blogs, nB, lane, [&](int i, int rank, double si) {
                if (rank == N - 1) s_thr = si;
            });
        }
        if (do_cand) {
            // --- ChooseNBestExpansions: joint top-N over the H*N per-hypothesis candidates, ranked the
            // same way: larger score first, then the earlier hypothesis, then the smaller token.  The N
            // candidates of a hypothesis arrive sorted by exactly that rule, hypotheses in order, so
            // "earlier place" decides equal scores.  (A place without a candidate holds NaN and never
            // compares as better.)
            sel_rank(s_key, nc, lane, [&](int c, int rank, double kc) {
                if (kc == kc && rank < N) s_sel[rank] = c;
            });
            if (pre_x) {
#pragma unroll
                for (int q = 0; q < SEL_PRE_FRAMES; ++q) s_xpre[q * WAVE + lane] = xpre[q];
            }
        }
        if (!do_finish) return;   // (the caller's barrier stands between the parts)
        sel_sync();
        // --- threshold test, in rank order: keep iff |B| < N or score > threshold (strict)
        const bool have_thr = s_have_thr != 0;
        const double thr = have_thr ? s_thr : 0.0;
        bool keep = false;   // lane r: the candidate of rank r becomes a hypothesis
        if (lane < N) {
            const int c = s_sel[lane];
            if (c >= 0) keep = (!have_thr) || (s_key[c] > thr);
        }
        if (drop) {
            if (lane == 0) {
                An.count[u] = 0;
                if (out) out->total = 0;
            }
        } else {
            // the kept candidates move up in rank order: place = kept candidates of better rank
            const u64 km = __ballot(keep);
            const int pos = __popcll(km & ((1ull << lane) - 1ull)), total = __popcll(km);
            if (lane == 0) {
                An.count[u] = total;
                if (out) out->total = total;
            }
            if (keep) {
                const int c = s_sel[lane];
                const int h = (int)(((float)c + 0.5f) * __builtin_amdgcn_rcpf((float)N));   // c / N for c < 256
                const int tok = s_ctok[c];
                const int slot_new = tbs_slot_id(u, parity, round, pos, d.R, N);
                const int pslot = s_aslot[h], pnode = s_anode[h];
                if (out) {
                    out->slot[pos] = slot_new;
                    out->pslot[pos] = pslot;
                    out->tok[pos] = tok;
                    out->pnode[pos] = pnode;
                    out->parent[pos] = h;
                }
                const long an = (long)u * N + pos;
                An.logs[an] = s_key[c];
                An.pnode[an] = pnode;
                if (!out) An.node[an] = -1;   // (a caller that takes `out` assigns the node itself)
                An.token[an] = tok;
                An.hash[an] = hash_append(s_ahash[h], tok);
                An.len[an] = s_alen[h] + 1;
                An.pslot[an] = pslot;
                An.slot[an] = slot_new;
                // d of the new hypothesis (Eq. 5 for the chosen token), normalised by its sum (Eq. 6)
                const int row0 = urow0 + h * (in.slot_rows ? d.S : sp);
                // (kept as logarithms: over a long segment d spans more than the range of float, and
                // the small entries matter to the next blank expansion)
                // The S' values wait in LDS (frame-major, so the lanes' accesses fall into different
                // banks) between the pass that reads the logits and the one that writes the normalised
                // result: going through the result array itself cost two more memory round trips.
                float *dh = An.dhat + an * d.S;
                if (pre_x) {
                    // (the S' <= 8 values stay in registers)
                    float x[SEL_PRE_FRAMES];
                    float mx = -INFINITY;
#pragma unroll
                    for (int q = 0; q < SEL_PRE_FRAMES; ++q) {
                        x[q] = s_xpre[q * WAVE + c] + in.lc[h * sp + min(q, sp - 1)];
                        if (q < sp) mx = fmaxf(mx, x[q]);
                    }
                    float sum = 0.f;
#pragma unroll
                    for (int q = 0; q < SEL_PRE_FRAMES; ++q)
                        if (q < sp) sum += __expf(x[q] - mx);
                    const float lz = mx + __logf(sum);
#pragma unroll
                    for (int q = 0; q < SEL_PRE_FRAMES; ++q)
                        if (q < d.S) dh[q] = q < sp ? x[q] - lz : -INFINITY;
                    for (int t = SEL_PRE_FRAMES; t < d.S; ++t) dh[t] = -INFINITY;
                } else if (logits) {
                    float *sd = s_dnew + lane;
                    float mx = -INFINITY;
                    for (int t0 = 0; t0 < sp; t0 += 8) {   // (eight logits asked for before the first is used)
                        float xv[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q) xv[q] = logits[(long)(row0 + min(t0 + q, sp - 1)) * d.V + tok];
#pragma unroll
                        for (int q = 0; q < 8; ++q)
                            if (t0 + q < sp) {
                                const float x = xv[q] + in.lc[h * sp + t0 + q];
                                sd[(t0 + q) * TBS_MAX_BEAM] = x;
                                mx = fmaxf(mx, x);
                            }
                    }
                    float sum = 0.f;
                    for (int t = 0; t < sp; ++t) sum += __expf(sd[t * TBS_MAX_BEAM] - mx);
                    const float lz = mx + __logf(sum);
                    for (int t = 0; t < sp; ++t) dh[t] = sd[t * TBS_MAX_BEAM] - lz;
                    for (int t = sp; t < d.S; ++t) dh[t] = -INFINITY;
                } else {
                    // (a caller without logits has segments of one frame: d normalised over one frame is (1))
                    dh[0] = 0.f;
                    for (int t = 1; t < d.S; ++t) dh[t] = -INFINITY;
                }
            }
        }
    }
}
