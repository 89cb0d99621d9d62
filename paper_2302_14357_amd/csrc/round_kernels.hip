// One round of the inner loop of Algorithm 1 behind the joiner, for small shapes, as one kernel:
// a workgroup per utterance expands all of the utterance's live hypotheses at once (Eq. 3-7 and the
// N best expansions of each, one team of 64 to 256 threads per hypothesis), hands the results to
// the select step through LDS, and that step does AddAndMerge, ChooseNthScore, the joint
// ChooseNBestExpansions with the threshold test and the new list A.  Where the workgroup has room for
// it the select step has a wave of its own, which stages B and A while the teams expand; behind the
// expansion it merges and finds the threshold while the workgroup's first wave ranks the candidates.
// Where the logits of one utterance's hypotheses (at most N * S' * V values) fit the registers of one
// workgroup this saves a kernel boundary and the trip of the candidates through memory in every
// round of a decode whose time is the length of its chain of dependent kernels.  What counts inside
// is the number of instructions per SIMD (a wave issues one every few cycles, the waves of a SIMD
// take turns) and the order of the requests to memory (they come back in order, and a wait behind a
// branch is a wait for all of them).
#include "expand_device.h"
#include "select_device.h"

__device__ __forceinline__ unsigned round_bf16(float f) {   // nearest, ties to even
    unsigned v = __float_as_uint(f);
    v += 0x7FFFu + ((v >> 16) & 1u);
    return v >> 16;
}

// S1NP > 0: segments of one frame (the standard breadth-first search, Eq. 1) in the slot layout.  The
// joiner GEMM kept no logits: `logits` points at its row partials (see PartEp), tiles_n per row, and
// the expansion of a hypothesis is the merge of its row's partials by one wave (TW = 1, SMAX = 1),
// lane l taking tile l with a list of up to S1NP candidates in registers.
template <int TW, int NV4, int SMAX, int S1NP>
__global__ void __launch_bounds__(1024)
k_round(Dims d, int round, int drop, const float *__restrict__ logits, AView A, AView An, BView B, RowView rv,
        int2 *nodes, float *__restrict__ row_stats, float *__restrict__ delta_nb, FixedView fx, int tiles_n) {
    constexpr int TT = TW * 64;
    typedef ExpandShared<SMAX, TW> TeamShared;
    extern __shared__ __attribute__((aligned(16))) unsigned char s_raw[];
    // LDS: the utterance's B list for the select step, one TeamShared per team, then what the teams
    // hand to the select step
    const int N = d.N;
    const size_t b_list = ((size_t)d.BCAP * (sizeof(double) + sizeof(u64) + 3 * sizeof(int)) + 15) & ~(size_t)15;
    TeamShared *teams = reinterpret_cast<TeamShared *>(s_raw + b_list);
    float *s_lc = reinterpret_cast<float *>(teams + (S1NP > 0 ? 0 : N));   // [H, S']
    float *s_dphi = s_lc + N * SMAX;                       // [H]
    float *s_cs = s_dphi + N;                              // [H, N]
    int *s_ct = reinterpret_cast<int *>(s_cs + N * N);     // [H, N]

    // Slot layout with a row range per XCD in the joiner GEMM: workgroup b runs on XCD b % 8 (workgroups
    // go to the XCDs in turn) and takes the (b / 8)-th utterance whose first joiner row lies in that
    // XCD's range, so that it finds the utterance's logits in its own XCD's L2.
    int u = blockIdx.x;
    if (fx.on && fx.xcd_rows > 0) {
        const int x = (int)blockIdx.x & 7, R = N * d.S;
        const int u0 = (x * fx.xcd_rows + R - 1) / R, u1 = ((x + 1) * fx.xcd_rows + R - 1) / R;
        u = u0 + ((int)blockIdx.x >> 3);
        if (u >= u1 || u >= d.U) return;   // (the whole workgroup, before any barrier)
    }
    const int team = __builtin_amdgcn_readfirstlane((int)threadIdx.x / TT), tid = (int)threadIdx.x % TT;
    // Where the workgroup has room for one more wave, that wave belongs to the select step: it stages
    // B and A in LDS while the teams expand, and goes on when they are done.  Otherwise the first
    // wave does the select step after its share of the expansion.
    const bool own_wave = (int)blockDim.x > N * TT;
    const bool sel_wave = own_wave ? (int)threadIdx.x >= N * TT : (int)threadIdx.x < WAVE;
    const int sel_lane = (int)threadIdx.x & 63;
    __shared__ SelectOut s_out;
    // Slot layout: everything the round has to know of the utterance lies side by side and comes
    // with one request.  What the kernel before this one wrote is asked for by the vector unit, a lane
    // per value, and handed to the scalar registers by lane reads: a request of the scalar unit for
    // memory that was written a moment ago was measured at ~1 us, one of the vector unit at a
    // quarter of that.
    SelectFigs fg;
    int used0 = 0, ncap = 0, nbase = 0;
    const int lane_w = (int)threadIdx.x & 63;
    const int team_c = team < N ? team : 0;   // (a team beyond N keeps its requests inside the utterance)
    int figv = 0;
    float doldv = 0.f, lbv = 0.f;
    if (fx.on) {
        figv = fx.fig[u * TBS_FIG_SIZE + (lane_w & (TBS_FIG_SIZE - 1))];
        if (S1NP == 0) {
            // (and, lane t, the hypothesis' d_old[t] and the blank logit of its frame t: rows that exist
            // whatever they hold)
            const int t = min(lane_w, d.S - 1);
            doldv = A.dhat[((long)u * N + team_c) * d.S + t];
            lbv = logits[((long)(u * N + team_c) * d.S + t) * d.V + d.blank];
        }
    } else {
        fg = select_figs(u, A, B, rv);
    }
    // Slot layout: where a hypothesis' logits lie follows from its place alone, so the teams ask for
    // them before anything is known about the utterance (all S rows of the place, or of the
    // utterance's first place for a team beyond N: memory that exists whatever it holds); what turns
    // out not to be a frame of a live hypothesis is cleared below.  The utterance's figures and the
    // logits then take one memory round trip together instead of two in a row.
    const bool early = S1NP == 0 && fx.on && !(own_wave && sel_wave);
    const int hslot = fx.on && fx.xh ? A.slot[(long)u * N + team_c] : 0;   // (of a hypothesis that may not exist)
    float e[SMAX][NV4 * 4];
    if (S1NP == 0 && early) expand_load<NV4, SMAX, TT>(e, logits, (u * N + team_c) * d.S, d.S, d.V, tid);
    if (fx.on) {
        fg.sp = __builtin_amdgcn_readlane(figv, TBS_FIG_SP);
        fg.cntA = __builtin_amdgcn_readlane(figv, TBS_FIG_CNT);
        fg.nB0 = __builtin_amdgcn_readlane(figv, TBS_FIG_NB);
        fg.parity = __builtin_amdgcn_readlane(figv, TBS_FIG_PAR);
        fg.urow0 = u * N * d.S;
        used0 = __builtin_amdgcn_readlane(figv, TBS_FIG_USED);
        ncap = __builtin_amdgcn_readlane(figv, TBS_FIG_CAP);
        nbase = __builtin_amdgcn_readlane(figv, TBS_FIG_BASE);
    }
    const int sp = fg.sp;
    const int H = sp > 0 ? fg.cntA : 0;
    if (H == 0) {   // (the same for the whole workgroup: nobody reaches a barrier)
        if (threadIdx.x == 0) An.count[u] = 0;
        if (fx.on) {
            if (threadIdx.x == 0) fx.fig[u * TBS_FIG_SIZE + TBS_FIG_CNT] = 0;
            if ((int)threadIdx.x < N) pair_mark_dead(rv, u * N + (int)threadIdx.x, u, d.S);
            if (threadIdx.x == 0) {
                if (u == 0) fx.live_sum[(fx.seq + 1) & 1] = 0;
                store_host(fx.host_live + (fx.seq & 1) * d.U + u, fx.seq << 8);
            }
        }
        return;
    }
    // (the utterance's pairs and rows follow each other: nothing is read from the pair list)
    const int pair0 = fx.on ? u * N : rv.utt_pair0[u], urow0 = fg.urow0;
    const bool live = team < H;
    SelectIn in;
    in.cand_score = s_cs;
    in.cand_tok = s_ct;
    in.dphi = s_dphi;
    in.lc = s_lc;
    in.slot_rows = fx.on;
    // Slot layout: the first LSTM layer's input rows of the hypotheses this round makes are bf16 copies
    // of their parents' h.  The parents are among this utterance's H hypotheses, so every team asks for
    // its own hypothesis' h now, beside the logits, and at the end writes it out once for every new
    // hypothesis made from it: the end of the kernel then has no memory round trip of its own.
    constexpr int HP = (160 + TT - 1) / TT;   // 16-byte pieces per thread for h up to 640 wide
    const int H4 = d.H >> 2;
    const bool pre_h = fx.on && fx.xh && H4 <= TT * HP;
    float4 hpar[HP];
    if (own_wave && sel_wave) {
        select_merge_utt(1, d, round, drop, u, sel_lane, logits, in, fg, A, An, B, rv, nodes, s_raw, &s_out);
        if constexpr (S1NP == 0) {
#pragma unroll
            for (int b = 0; b < EXPAND_PAIR_BARRIERS; ++b) __syncthreads();
        }
    } else if constexpr (S1NP > 0) {
        if (pre_h && live) {
            const long slot = A.slot[(long)u * N + team];
#pragma unroll
            for (int q = 0; q < HP; ++q)
                hpar[q] = reinterpret_cast<const float4 *>(fx.pool_h + slot * d.H)[min(tid + TT * q, H4 - 1)];
        }
        // Every request is made whatever the lane's tile and the team's hypothesis are (addresses
        // clamped to ones that exist); what does not exist is masked afterwards.
        const int pw = part_width(N), hyp = live ? team : 0;
        const float *p = logits + ((long)(pair0 + hyp) * tiles_n + min(tid, tiles_n - 1)) * pw;   // (S = 1: a pair's row is its place)
        const float la = A.dhat[((long)u * N + hyp) * d.S];   // log d_old[1]: alpha_1 of Eq. 3
        const float4 hd = *reinterpret_cast<const float4 *>(p);
        float lv[S1NP];
        int lk[S1NP];
#pragma unroll
        for (int n = 0; n < S1NP; ++n) {
            lv[n] = p[4 + min(n, N - 1)];
            lk[n] = __float_as_int(p[4 + N + min(n, N - 1)]);
        }
        const bool have = live && tid < tiles_n;
#pragma unroll
        for (int n = 0; n < S1NP; ++n)
            if (!have || n >= N || lk[n] < 0) {
                lv[n] = -INFINITY;
                lk[n] = 0x7fffffff;
            }
        const float mt = have ? hd.x : -INFINITY;
        const float m = wave_max_ord(mt);
        const float z = wave_sum(mt > -INFINITY ? hd.y * __expf(mt - m) : 0.f);
        const float lb = wave_max_ord(have ? hd.z : -INFINITY);
        // Eq. 1: an expansion's score relative to the hypothesis is the token's (or blank's) log
        // probability at the frame (plus log alpha_1 = log d_old[1], which is 0 for a normalised d)
        const float base = la - m - __logf(z);
        if (tid == 0 && live) {
            s_dphi[team] = base + lb;
            s_lc[team] = base;
        }
        for (int n = 0; n < N; ++n) {   // the N best of the row: N rounds of arg-max over the lists' heads
            float bv = lv[0];
            int bk = lk[0];
            wave_argmax(bv, bk);
            const bool ok = bv > -INFINITY;
            if (tid == 0 && live) {
                s_cs[team * N + n] = ok ? base + bv : -INFINITY;
                s_ct[team * N + n] = ok ? bk : -1;
            }
            if (ok && lk[0] == bk) {   // (a token lies in one tile: one lane's list moves up)
#pragma unroll
                for (int i = 0; i + 1 < S1NP; ++i) {
                    lv[i] = lv[i + 1];
                    lk[i] = lk[i + 1];
                }
                lv[S1NP - 1] = -INFINITY;
                lk[S1NP - 1] = 0x7fffffff;
            }
        }
    } else {
        ExpandPair<SMAX> pi;
        if (live && early) {
            pi.pair = pair0 + team;
            pi.row0 = urow0 + team * d.S;
            pi.sp = sp;
#pragma unroll
            for (int t = 0; t < SMAX; ++t) {
                pi.dold[t] = t < sp ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(doldv), t)) : -INFINITY;
                pi.lblank[t] = t < sp ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(lbv), t)) : 0.f;
            }
        } else if (live) {
            expand_pair_info_at(pi, pair0 + team, urow0 + team * (fx.on ? d.S : sp), sp, u, team, d, A, logits);
        } else {   // a team without a hypothesis reads the utterance's first row and scores nothing
            pi.pair = pair0;
            pi.row0 = urow0;
            pi.sp = 0;
#pragma unroll
            for (int t = 0; t < SMAX; ++t) {
                pi.dold[t] = -INFINITY;
                pi.lblank[t] = 0.f;
            }
        }
        if (!early) {
            expand_load<NV4, SMAX, TT>(e, logits, pi.row0, pi.sp, d.V, tid);
        } else {
#pragma unroll
            for (int t = 0; t < SMAX; ++t)
                if (t >= pi.sp) {   // (uniform) not a frame: whatever was read, it must be a number
#pragma unroll
                    for (int c = 0; c < NV4 * 4; ++c) e[t][c] = 0.f;
                }
        }
        expand_pair<NV4, SMAX, TT>(e, pi, teams[team], d, tid, live, s_lc + team * sp, s_dphi + team, s_cs + team * N,
                                   s_ct + team * N, row_stats, delta_nb);
    }
    __syncthreads();
    // (the parent's h is asked for only now, by the state slot asked for at the start: requests made
    // beside those for the logits would have to be waited for with them, two round trips in a row;
    // here the row's trip runs while the select step works)
    if (S1NP == 0 && pre_h && live && !(own_wave && sel_wave)) {
        const long slot = hslot;
#pragma unroll
        for (int q = 0; q < HP; ++q)
            hpar[q] = reinterpret_cast<const float4 *>(fx.pool_h + slot * d.H)[min(tid + TT * q, H4 - 1)];
    }
    // Behind the expansion the select step has two parts that need nothing of each other: the select
    // wave merges the blank expansions into B and finds the threshold while the workgroup's first wave,
    // idle by now, ranks the candidates; the select wave goes on when both are done.
    const float *lg = S1NP > 0 ? nullptr : logits;   // (no logits: d of a new hypothesis over one frame is (1))
    if (own_wave) {
        if (sel_wave)
            select_merge_utt(4, d, round, drop, u, sel_lane, lg, in, fg, A, An, B, rv, nodes, s_raw, &s_out);
        else if ((int)threadIdx.x < WAVE)
            select_merge_utt(3, d, round, drop, u, sel_lane, lg, in, fg, A, An, B, rv, nodes, s_raw, &s_out);
        __syncthreads();
    }
    if (sel_wave) {
        select_merge_utt(own_wave ? 5 : 0, d, round, drop, u, sel_lane, lg, in, fg, A, An, B, rv, nodes, s_raw, &s_out);
        if (fx.on) {
            // Slot layout: what a row list kernel would do for this utterance.  The new hypotheses
            // take trie nodes from the utterance's own range, their pairs get their descriptors, the
            // places of A beyond them are marked dead, and the host hears how many there are.
            sel_sync();
            const int lane = sel_lane, total = s_out.total;
            bool full = false;
            if (lane < N) {
                const int j = u * N + lane;
                if (lane < total) {
                    const int tok = s_out.tok[lane];
                    full = used0 + lane >= ncap;
                    const int node = full ? 0 : nbase + used0 + lane;
                    if (!full) nodes[node] = make_int2(s_out.pnode[lane], tok);
                    An.node[j] = node;
                    rv.pair_u[j] = u;
                    rv.pair_h[j] = lane;
                    rv.pair_row0[j] = j * d.S;
                    rv.pair_len[j] = sp;
                    rv.pair_slot[j] = s_out.slot[lane];
                    rv.pair_pslot[j] = s_out.pslot[lane];
                    rv.pair_frame0[j] = fx.utt_off[u] + fx.seg * d.S;
                    rv.pair_tok[j] = tok;
                } else {
                    pair_mark_dead(rv, j, u, d.S);
                }
            }
            const bool any_full = __ballot(full) != 0;
            if (lane == 0) {
                rv.utt_par[u] = fg.parity;   // (the kernel that started the segment may have left this to the round)
                int *fig = fx.fig + u * TBS_FIG_SIZE;
                fig[TBS_FIG_CNT] = total;
                fig[TBS_FIG_NB] = s_out.nB;
                fig[TBS_FIG_USED] = min(used0 + total, ncap);
                if (total) atomicAdd(fx.live_sum + (fx.seq & 1), total);
                if (u == 0) fx.live_sum[(fx.seq + 1) & 1] = 0;
                store_host(fx.host_live + (fx.seq & 1) * d.U + u, (fx.seq << 8) | (any_full ? 64 : 0) | total);
            }
        }
    }
    if (pre_h) {
        __syncthreads();
        const int total = s_out.total;
        if (live) {
            uint2 hb[HP];
#pragma unroll
            for (int q = 0; q < HP; ++q)
                hb[q] = make_uint2((unsigned)round_bf16(hpar[q].x) | ((unsigned)round_bf16(hpar[q].y) << 16),
                                   (unsigned)round_bf16(hpar[q].z) | ((unsigned)round_bf16(hpar[q].w) << 16));
            for (int i = 0; i < total; ++i)
                if (s_out.parent[i] == team) {
#pragma unroll
                    for (int q = 0; q < HP; ++q)
                        if (tid + TT * q < H4) reinterpret_cast<uint2 *>(fx.xh)[(long)(u * N + i) * H4 + tid + TT * q] = hb[q];
                }
        }
    } else if (fx.on && fx.xh) {
        // (h too wide to wait in registers: read the parents' rows now)
        __syncthreads();
        const int total = s_out.total;
        for (int idx = (int)threadIdx.x; idx < total * H4; idx += (int)blockDim.x) {
            const int h = idx / H4, i = idx - h * H4;
            const float4 v = reinterpret_cast<const float4 *>(fx.pool_h + (long)s_out.pslot[h] * d.H)[i];
            reinterpret_cast<uint2 *>(fx.xh)[(long)(u * N + h) * H4 + i] =
                make_uint2((unsigned)round_bf16(v.x) | ((unsigned)round_bf16(v.y) << 16),
                           (unsigned)round_bf16(v.z) | ((unsigned)round_bf16(v.w) << 16));
        }
    }
}

// which instantiation serves the shape (0 = none): a hypothesis' S x V logits stay within the
// registers of its team.  A team is one wave whatever the beam (measured, ms per decode of the
// Librispeech-like batch at S = 3 with teams of 4 / 2 / 1 waves: N = 2: 16.6 / 16.9 / 16.6, N = 4:
// 19.1 / 17.6 / 17.4, N = 5: - / 18.2 / 18.0, N = 8: - / 28.3 / 26.4): what a wave more per hypothesis saves in
// values per thread it costs in reductions, candidate lists and their merge, and the waves of a
// workgroup share four SIMDs.  The template keeps teams of several waves.
static int round_variant(const Dims &d) {
    if (d.V % 4 || d.S > 5 || d.N > 16) return 0;
    const int v4 = d.V / 4;
    const int nv4 = v4 <= 64 ? 1 : (v4 <= 128 ? 2 : 4);
    if (v4 > 64 * nv4) return 0;
    return nv4 * 10 + (d.S <= 3 ? 3 : 5);
}

bool round_fits(const Dims &d) { return round_variant(d) != 0; }

template <int TW, int NV4, int SMAX, int S1NP = 0>
static hipError_t round_launch(hipStream_t st, const Dims &d, int round, int drop, const float *logits, AView A,
                               AView An, BView B, RowView rv, int2 *nodes, float *row_stats, float *delta_nb,
                               const FixedView &fx, int tiles_n = 0) {
    const size_t b_list = ((size_t)d.BCAP * (sizeof(double) + sizeof(u64) + 3 * sizeof(int)) + 15) & ~(size_t)15;
    const size_t shm = b_list + (S1NP > 0 ? 0 : (size_t)d.N * sizeof(ExpandShared<SMAX, TW>)) +
                       sizeof(float) * ((size_t)d.N * SMAX + d.N + 2 * (size_t)d.N * d.N);
    static size_t attr_for = 0;
    if (shm > attr_for) {   // (static LDS of the select step comes on top: raise the limit to what the launch needs)
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_round<TW, NV4, SMAX, S1NP>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) return e;
        attr_for = shm;
    }
    // (one wave more for the select step where 1024 threads allow it)
    const int threads = d.N * TW * 64 + (d.N * TW * 64 + 64 <= 1024 ? 64 : 0);
    // (with a row range per XCD: eight workgroups, one per XCD, for each place in the longest XCD's list)
    const int grid = fx.on && fx.xcd_rows > 0 ? 8 * (fx.xcd_rows / (d.N * d.S) + 1) : d.U;
    hipLaunchKernelGGL((k_round<TW, NV4, SMAX, S1NP>), dim3(grid), dim3(threads), shm, st, d, round, drop, logits, A, An,
                       B, rv, nodes, row_stats, delta_nb, fx, tiles_n);
    return hipGetLastError();
}

hipError_t launch_round(hipStream_t st, const Dims &d, int round, int drop, const float *logits, AView A, AView An,
                        BView B, RowView rv, int2 *nodes, float *row_stats, float *delta_nb, const FixedView *fxp) {
    FixedView fx{};
    if (fxp) fx = *fxp;
    if (fx.on && fx.xh && (d.H & 3)) return hipErrorInvalidValue;
    switch (round_variant(d)) {
        case 13: return round_launch<1, 1, 3>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb, fx);
        case 15: return round_launch<1, 1, 5>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb, fx);
        case 23: return round_launch<1, 2, 3>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb, fx);
        case 25: return round_launch<1, 2, 5>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb, fx);
        case 43: return round_launch<1, 4, 3>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb, fx);
        case 45: return round_launch<1, 4, 5>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb, fx);
        default: return hipErrorInvalidValue;
    }
}

bool round_s1_fits(const Dims &d) { return d.S == 1 && d.N >= 1 && d.N <= 16 && (d.V + 63) / 64 <= 64 && (d.H & 3) == 0; }

hipError_t launch_round_s1(hipStream_t st, const Dims &d, int round, int drop, const float *part, int tiles_n, AView A,
                           AView An, BView B, RowView rv, int2 *nodes, const FixedView *fxp) {
    if (!fxp || !fxp->on || !part || !round_s1_fits(d) || tiles_n < 1 || tiles_n > 64) return hipErrorInvalidValue;
    if (d.N <= 4) return round_launch<1, 1, 1, 4>(st, d, round, drop, part, A, An, B, rv, nodes, nullptr, nullptr, *fxp, tiles_n);
    if (d.N <= 8) return round_launch<1, 1, 1, 8>(st, d, round, drop, part, A, An, B, rv, nodes, nullptr, nullptr, *fxp, tiles_n);
    return round_launch<1, 1, 1, 16>(st, d, round, drop, part, A, An, B, rv, nodes, nullptr, nullptr, *fxp, tiles_n);
}
