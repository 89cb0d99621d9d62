// Beam bookkeeping kernels of token-wise RNN-T beam search (Algorithm 1):
// ChooseNBest at the head of a segment, the row list of a joiner call,
// AddAndMerge / ChooseNthScore / ChooseNBestExpansions with the threshold
// test, and reading the N-best out of the token trie.
//
// One 64-lane wavefront owns one utterance, so every list operation of the
// algorithm is a few lane-parallel passes and nothing needs a grid-wide
// barrier.  Token sequences live in a trie of (parent, token) nodes; a
// hypothesis carries its node, length and a 64-bit hash; two hypotheses are
// "the same tokens" when hash and length agree and a walk up the trie agrees.
#include "tbs_internal.h"
#include "select_device.h"

// ------------------------------------------------------------------ batch init
__global__ void k_init_batch(Dims d, BView B, AView A0, AView A1, RowView rv, int2 *nodes, float *pool_p,
                             float *pool_h, float *pool_c, const float *pred_init, long pool_rows) {
    int u = blockIdx.x;
    int tid = threadIdx.x;
    // B = [([], 1, InitPredictor(), Null)]: the empty sequence is trie node 0;
    // its predictor state sits in the "previous segment" arena (parity 1).
    int slot = tbs_slot_id(u, 1, 0, 0, d.R, d.N);
    if (tid == 0) {
        B.count[u] = 1;
        B.logs[(long)u * d.BCAP] = 0.0;
        B.node[(long)u * d.BCAP] = 0;
        B.hash[(long)u * d.BCAP] = 0ull;
        B.len[(long)u * d.BCAP] = 0;
        B.slot[(long)u * d.BCAP] = slot;
        A0.count[u] = 0;
        A1.count[u] = 0;
        rv.utt_sp[u] = 0;
        rv.utt_pair0[u] = 0;
        rv.utt_par[u] = 1;
        if (u == 0) {
            nodes[0] = make_int2(-1, -1);
            rv.counts[TBS_CNT_PAIRS] = 0;
            rv.counts[TBS_CNT_ROWS] = 0;
            rv.counts[TBS_CNT_NODES] = 1;
            rv.counts[TBS_CNT_ERR] = 0;
            rv.counts[TBS_CNT_UTTS] = 0;
            rv.counts[TBS_CNT_FRAMES] = 0;
            rv.counts[TBS_CNT_SEQ] = 0;
            rv.counts[TBS_CNT_NODE_BASE] = 1;
            rv.counts[TBS_CNT_ACC_CALLS] = 0;
            rv.counts[TBS_CNT_ACC_JOINED] = 0;
        }
    }
    for (int j = tid; j < d.Dj; j += blockDim.x) pool_p[(long)slot * d.Dj + j] = pred_init[j];
    for (int l = 0; l < d.L; ++l)
        for (int j = tid; j < d.H; j += blockDim.x) {
            pool_h[((long)l * pool_rows + slot) * d.H + j] = 0.f;
            pool_c[((long)l * pool_rows + slot) * d.H + j] = 0.f;
        }
}

hipError_t launch_init_batch(hipStream_t st, const Dims &d, BView B, AView A0, AView A1, RowView rv, int2 *nodes,
                             float *pool_p, float *pool_h, float *pool_c, const float *pred_init,
                             long pool_rows) {
    hipLaunchKernelGGL(k_init_batch, dim3(d.U), dim3(256), 0, st, d, B, A0, A1, rv, nodes, pool_p, pool_h, pool_c,
                       pred_init, pool_rows);
    return hipGetLastError();
}

// ------------------------------------------------------------------ segment head
// A = ChooseNBest(B); B = []; d = (s, 0, ..., 0)   (Algorithm 1, head of the outer loop)
// The workgroup ranks B and writes A; then it moves the survivors' predictor state into this
// segment's arena (slot r=0): the arena of the segment before last is reused, and a survivor may have
// been carried, untouched, from there.  In the slot layout it also forms the joiner input rows of the
// segment's first round, act(e_t + p) as bf16 (Section 3.1), from the p values it is moving.
// A SIMD issues an instruction of one of its waves every few cycles, so what counts in a kernel of
// this size is the number of instructions per SIMD: a workgroup is four waves, one per SIMD, and in
// the slot layout, where a small batch leaves most of the chip idle, `parts` workgroups share an
// utterance: each ranks B for itself (a few hundred instructions) and moves its share of the
// survivors' rows, a 16-byte piece of one row per thread; the first also writes A and the
// descriptors.  With parts > 1 nothing that the other workgroups of the utterance still have to read
// is changed here: B's count and the arena flag are left to the round kernel that follows.
__device__ __forceinline__ unsigned seg_bf16(float f) {   // nearest, ties to even
    unsigned v = __float_as_uint(f);
    v += 0x7FFFu + ((v >> 16) & 1u);
    return v >> 16;
}
#define SEG_THREADS 256
#define SEG_ENC_LOADS ((TBS_FIXED_SMAX * 1024 / 4 + SEG_THREADS - 1) / SEG_THREADS)   // 8-byte pieces of S rows of up to 1024 columns, per thread
__global__ void __launch_bounds__(SEG_THREADS)
k_segment_begin(Dims d, int seg, const int *utt_T, BView B, AView A, RowView rv, float *pool_p,
                float *pool_h, float *pool_c, long pool_rows, FixedView fx) {
    __shared__ int s_src[TBS_MAX_BEAM], s_dst[TBS_MAX_BEAM];
    __shared__ int s_n;
    __shared__ uint2 s_enc[TBS_FIXED_SMAX * 1024 / 4];   // the segment's frames, [frame][4 columns]
    const int parts = fx.parts > 1 ? fx.parts : 1;
    const int u = blockIdx.x / parts, part = blockIdx.x - u * parts, tid = threadIdx.x;
    const bool first = part == 0;
    // Everything the head of the kernel needs is requested at once, before anything is known:
    // the utterance's figures and, per thread, one entry of B (the first SEG_THREADS entries
    // cover every list but the very longest), so that the ranking below starts after one memory
    // round trip instead of four.
    __shared__ double s_bl[2048];           // BCAP is at most 2048
    const long bb = (long)u * d.BCAP;
    const int e0 = min(tid, d.BCAP - 1);
    const int T_u = utt_T[u], nB = B.count[u], par_old = rv.utt_par[u];
    const double my_logs = B.logs[bb + e0];
    const int my_slot = B.slot[bb + e0], my_node = B.node[bb + e0], my_len = B.len[bb + e0];
    const u64 my_hash = B.hash[bb + e0];
    int left = T_u - seg * d.S;
    int sp = left < 0 ? 0 : (left > d.S ? d.S : left);
    // The frames of the segment come from memory nobody has touched yet, the slowest request of the
    // kernel: they are asked for now, behind the entries of B (requests come back in order), and wait
    // in registers until the ranking is done.  Asked for whether wanted or not, from an address that
    // exists in either case: a request behind a condition would make every later wait a wait for all.
    const bool rows_here = fx.on && fx.amat != nullptr && sp > 0;
    const int cp = d.Dj >> 2;   // pieces of four columns in a row
    uint2 ev[SEG_ENC_LOADS];
    {
        const bf16_t *ebase = rows_here ? fx.enc + ((long)fx.utt_off[u] + (long)seg * d.S) * d.Dj
                                        : reinterpret_cast<const bf16_t *>(pool_p);
        const int pieces = rows_here ? sp * cp : 1;
#pragma unroll
        for (int q = 0; q < SEG_ENC_LOADS; ++q)
            ev[q] = reinterpret_cast<const uint2 *>(ebase)[min(tid + q * SEG_THREADS, pieces - 1)];   // (rows follow each other)
    }
    if (tid == 0) {
        if (first) rv.utt_sp[u] = sp;
        s_n = 0;
    }
    if (fx.on && tid == 0 && first) {
        rv.utt_pair0[u] = u * d.N;
        rv.utt_row0[u] = u * d.N * d.S;
        if (u == 0) fx.live_sum[(fx.seq + 1) & 1] = 0;   // the counter of the launch after this one
    }
    if (sp == 0) {  // finished (or empty) utterance: B keeps the final list
        if (!first) return;
        if (tid == 0) A.count[u] = 0;
        if (fx.on) {
            if (tid == 0) {
                int *fig = fx.fig + u * TBS_FIG_SIZE;
                fig[TBS_FIG_SP] = 0;
                fig[TBS_FIG_CNT] = 0;
            }
            if (tid < d.N) pair_mark_dead(rv, u * d.N + tid, u, d.S);
            if (tid == 0) store_host(fx.host_live + (fx.seq & 1) * d.U + u, fx.seq << 8);
        }
        return;
    }
    const int parity = par_old ^ 1;   // the arena the survivors are not in
    // the scores go through LDS: ranking by counting reads every score once per entry
    if (tid < nB) s_bl[tid] = my_logs;
    for (int i = tid + SEG_THREADS; i < nB; i += SEG_THREADS) s_bl[i] = B.logs[bb + i];
    __syncthreads();
    for (int i = tid; i < nB; i += SEG_THREADS) {
        const double si = s_bl[i];
        int rank = 0;
        for (int j = 0; j < nB; ++j) {
            const double sj = s_bl[j];
            rank += (sj > si) || (sj == si && j < i);
        }
        if (rank < d.N) {
            const long a = (long)u * d.N + rank, b = bb + i;
            const bool mine = i == tid;
            const int src = mine ? my_slot : B.slot[b], dst = tbs_slot_id(u, parity, 0, rank, d.R, d.N);
            s_src[rank] = src;
            s_dst[rank] = dst;
            if (first) {
                A.logs[a] = si;
                A.node[a] = mine ? my_node : B.node[b];
                A.hash[a] = mine ? my_hash : B.hash[b];
                A.len[a] = mine ? my_len : B.len[b];
                A.pslot[a] = src;
                A.slot[a] = dst;
                A.pnode[a] = -1;
                A.token[a] = -1;
                float *dh = A.dhat + a * d.S;
                dh[0] = 0.f;   // d = (s, 0, ..., 0), normalised and as logarithms
                for (int t = 1; t < d.S; ++t) dh[t] = -INFINITY;
            }
        }
    }
    if (tid == 0) {
        if (first) A.count[u] = nB < d.N ? nB : d.N;
        s_n = nB < d.N ? nB : d.N;
    }
    if (rows_here) {
#pragma unroll
        for (int q = 0; q < SEG_ENC_LOADS; ++q)
            if (tid + q * SEG_THREADS < sp * cp) s_enc[tid + q * SEG_THREADS] = ev[q];
    }
    __syncthreads();
    if (tid == 0 && parts == 1) {   // (every thread has read the old values by now)
        rv.utt_par[u] = parity;
        B.count[u] = 0;
    }
    if (fx.on && first) {   // slot layout: this utterance's pair descriptors for the first round, its count to the host
        const int cnt = s_n;
        if (tid < d.N) {
            const int j = u * d.N + tid;
            if (tid < cnt) {
                rv.pair_u[j] = u;
                rv.pair_h[j] = tid;
                rv.pair_row0[j] = j * d.S;
                rv.pair_len[j] = sp;
                rv.pair_slot[j] = s_dst[tid];
                rv.pair_pslot[j] = s_src[tid];
                rv.pair_frame0[j] = fx.utt_off[u] + seg * d.S;
                rv.pair_tok[j] = -1;
            } else {
                pair_mark_dead(rv, j, u, d.S);
            }
        }
        if (tid == 0) {
            int *fig = fx.fig + u * TBS_FIG_SIZE;
            fig[TBS_FIG_SP] = sp;
            fig[TBS_FIG_CNT] = cnt;
            fig[TBS_FIG_NB] = 0;
            fig[TBS_FIG_PAR] = parity;
            atomicAdd(fx.live_sum + (fx.seq & 1), cnt);
            store_host(fx.host_live + (fx.seq & 1) * d.U + u, (fx.seq << 8) | cnt);
        }
    }
    // The survivors' predictor outputs and LSTM states move to their new slots: item (survivor k,
    // piece j) moves piece j (16 bytes where the widths allow) of the survivor's output row and of
    // its h and c rows of every layer, all requested before the first is stored.
    const int n = s_n;
    auto copy_all = [&](auto unit_tag, int w) {   // w = floats per unit
        using UNIT = decltype(unit_tag);
        const int up = d.Dj / w, uh = d.H / w, widest = max(up, uh);
        const float rcp_w = __builtin_amdgcn_rcpf((float)widest);   // (item / widest exactly, items < 2^16)
        for (int it = part * SEG_THREADS + tid; it < n * widest; it += parts * SEG_THREADS) {
            const int k = (int)(((float)it + 0.5f) * rcp_w), j = it - k * widest;
            const long src = s_src[k], dst = s_dst[k];
            const int jp = min(j, up - 1), jh = min(j, uh - 1);
            const UNIT vp = reinterpret_cast<const UNIT *>(pool_p + src * d.Dj)[jp];
            UNIT vh[TBS_MAX_LAYERS], vc[TBS_MAX_LAYERS];
#pragma unroll
            for (int l = 0; l < TBS_MAX_LAYERS; ++l)
                if (l < d.L) {   // (uniform)
                    vh[l] = reinterpret_cast<const UNIT *>(pool_h + ((long)l * pool_rows + src) * d.H)[jh];
                    vc[l] = reinterpret_cast<const UNIT *>(pool_c + ((long)l * pool_rows + src) * d.H)[jh];
                }
            if (j < up) reinterpret_cast<UNIT *>(pool_p + dst * d.Dj)[j] = vp;
            if (j < uh) {
#pragma unroll
                for (int l = 0; l < TBS_MAX_LAYERS; ++l)
                    if (l < d.L) {
                        reinterpret_cast<UNIT *>(pool_h + ((long)l * pool_rows + dst) * d.H)[j] = vh[l];
                        reinterpret_cast<UNIT *>(pool_c + ((long)l * pool_rows + dst) * d.H)[j] = vc[l];
                    }
            }
            if constexpr (sizeof(UNIT) == 16) {
                if (rows_here && j < up) {
                    // (hypothesis k of the utterance is pair u*N + k: rows from pair * S)
                    const float p4[4] = {vp.x, vp.y, vp.z, vp.w};
                    uint2 *arow = reinterpret_cast<uint2 *>(fx.amat + (long)(u * d.N + k) * d.S * d.Dj) + j;
                    for (int t = 0; t < sp; ++t) {
                        const uint2 e2 = s_enc[t * cp + j];
                        const float e4[4] = {__uint_as_float(e2.x << 16), __uint_as_float(e2.x & 0xFFFF0000u),
                                             __uint_as_float(e2.y << 16), __uint_as_float(e2.y & 0xFFFF0000u)};
                        unsigned o[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) o[q] = seg_bf16(tbs_joiner_act(e4[q] + p4[q], fx.act));
                        arow[(long)t * cp] = make_uint2(o[0] | (o[1] << 16), o[2] | (o[3] << 16));
                    }
                }
            }
        }
    };
    if (((d.Dj | d.H) & 3) == 0) copy_all(float4{}, 4);
    else copy_all(float{}, 1);
}

hipError_t launch_segment_begin(hipStream_t st, const Dims &d, int seg, const int *utt_T, BView B,
                                AView A, RowView rv, float *pool_p, float *pool_h, float *pool_c, long pool_rows,
                                const FixedView *fx) {
    FixedView f{};
    if (fx) f = *fx;
    if (f.parts > 1 && !f.on) return hipErrorInvalidValue;   // (only the slot layout's round kernel finishes what the parts leave)
    hipLaunchKernelGGL(k_segment_begin, dim3(d.U * (f.parts > 1 ? f.parts : 1)), dim3(SEG_THREADS), 0, st, d, seg, utt_T, B, A, rv, pool_p,
                       pool_h, pool_c, pool_rows, f);
    return hipGetLastError();
}

// ------------------------------------------------------------------ row list
// The joiner rows of a round are the (pair, frame) combinations of the live
// (utterance, hypothesis) pairs, compacted.  One workgroup (a wave) per
// utterance: each reads the counts of ALL utterances, which the kernel before it
// wrote, and sums those ahead of its own, so no workgroup waits for another and
// nothing travels between them; it then fills its pairs and rows and gives new
// hypotheses their trie nodes.  The first workgroup also owns the totals: it
// publishes them to the host, with the number of this launch last, before it
// fills anything.
__device__ __forceinline__ int wave_sum_int(int v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

__device__ __forceinline__ void rowfill_lists(const Dims &d, int seg, const int *utt_off, AView A, RowView rv, int2 *nodes,
                                              int assign_nodes, int *host_counts, int seq, int u, int lane, bool share,
                                              int *s_pslot, int *s_pair0, int *s_cnt) {
    // trie nodes handed out so far: launches alternate between two slots, so that the first
    // workgroup can store the new figure while others still read the old one
    const int slot_old = (seq & 1) ? TBS_CNT_NODE_BASE : TBS_CNT_NODES;
    const int slot_new = (seq & 1) ? TBS_CNT_NODES : TBS_CNT_NODE_BASE;
    const int node_base = rv.counts[slot_old];
    const int frame0 = utt_off[u] + seg * d.S;
    // what the fill below needs of this utterance's hypotheses, lane h holding hypothesis h:
    // requested together with the counts, so the kernel costs one memory round trip, not two
    const long ah = (long)u * d.N + min(lane, d.N - 1);
    const int h_slot = A.slot[ah], h_pslot = A.pslot[ah], h_tok = A.token[ah], h_pnode = A.pnode[ah];
    int before_p = 0, before_r = 0, tot_p = 0, tot_r = 0, utts = 0, frames = 0, my_sp = 0, my_cnt = 0;
    for (int base = 0; base < d.U; base += WAVE) {
        const int v = base + lane;
        const int sp = v < d.U ? rv.utt_sp[v] : 0;
        const int c = (v < d.U && sp > 0) ? A.count[v] : 0;
        const int r = c * sp;
        if (v < u) { before_p += c; before_r += r; }
        if (v == u) { my_sp = sp; my_cnt = c; }
        tot_p += c;
        tot_r += r;
        utts += c > 0;
        frames += c > 0 ? sp : 0;
    }
    const int pair0 = wave_sum_int(before_p), row0 = wave_sum_int(before_r);
    const int sp = wave_sum_int(my_sp), cnt = wave_sum_int(my_cnt);
    if (u == 0) {
        tot_p = wave_sum_int(tot_p);
        tot_r = wave_sum_int(tot_r);
        utts = wave_sum_int(utts);
        frames = wave_sum_int(frames);
        if (lane == 0) {
            int err = rv.counts[TBS_CNT_ERR];
            int nodes_used = node_base;
            if (assign_nodes) {
                nodes_used = node_base + tot_p;
                if (nodes_used > d.max_nodes) { err |= TBS_ERRF_NODES; nodes_used = d.max_nodes; }
            }
            // every row list is followed by one joiner call over its rows: the counters of Section
            // 4.2 (invocations, frames joined; per utterance summed) are kept here, so that the host
            // need not see every row list
            const int acc_calls = rv.counts[TBS_CNT_ACC_CALLS] + utts, acc_joined = rv.counts[TBS_CNT_ACC_JOINED] + frames;
            rv.counts[TBS_CNT_ACC_CALLS] = acc_calls;
            rv.counts[TBS_CNT_ACC_JOINED] = acc_joined;
            if (host_counts) {
                store_host(host_counts + TBS_CNT_ACC_CALLS, acc_calls);
                store_host(host_counts + TBS_CNT_ACC_JOINED, acc_joined);
                store_host(host_counts + TBS_CNT_PAIRS, tot_p);
                store_host(host_counts + TBS_CNT_ROWS, tot_r);
                store_host(host_counts + TBS_CNT_NODES, nodes_used);
                store_host(host_counts + TBS_CNT_ERR, err);
                store_host(host_counts + TBS_CNT_UTTS, utts);
                store_host(host_counts + TBS_CNT_FRAMES, frames);
                __builtin_amdgcn_s_waitcnt(0);   // the figures are acknowledged before their number goes out
                store_host(host_counts + TBS_CNT_SEQ, seq);
            }
            rv.counts[TBS_CNT_PAIRS] = tot_p;
            rv.counts[TBS_CNT_ROWS] = tot_r;
            rv.counts[slot_new] = nodes_used;
            rv.counts[TBS_CNT_ERR] = err;
            rv.counts[TBS_CNT_UTTS] = utts;
            rv.counts[TBS_CNT_FRAMES] = frames;
        }
    }
    if (lane == 0) {
        rv.utt_pair0[u] = pair0;
        rv.utt_row0[u] = row0;
    }
    for (int base = 0; base < cnt * sp; base += WAVE) {   // (cnt and sp are the same in every lane)
        const int idx = base + lane;
        const bool valid = idx < cnt * sp;
        const int h = valid ? idx / sp : 0, t = idx - h * sp;
        // every lane takes part in the exchanges, whatever it does with the result
        const int slot = __shfl(h_slot, h), pslot = __shfl(h_pslot, h), tok = __shfl(h_tok, h),
                  pnode = __shfl(h_pnode, h);
        if (!valid) continue;
        const long a = (long)u * d.N + h;
        rv.row_enc[row0 + idx] = frame0 + t;
        rv.row_slot[row0 + idx] = slot;
        if (t == 0) {
            const int j = pair0 + h;
            rv.pair_u[j] = u;
            rv.pair_h[j] = h;
            rv.pair_row0[j] = row0 + h * sp;
            rv.pair_len[j] = sp;
            rv.pair_slot[j] = slot;
            rv.pair_pslot[j] = pslot;
            rv.pair_frame0[j] = frame0;
            rv.pair_tok[j] = tok;
            if (assign_nodes) {
                const int node = node_base + j;
                if (node < d.max_nodes) {
                    nodes[node] = make_int2(pnode, tok);
                    A.node[a] = node;
                } else {
                    A.node[a] = 0;
                }
            }
        }
    }
    if (share) {   // for the other waves of the workgroup
        if (lane < d.N) s_pslot[lane] = h_pslot;
        if (lane == 0) {
            *s_pair0 = pair0;
            *s_cnt = cnt;
        }
    }
}

// With gather_h not null the workgroup has four waves: the first does all of the above, then all
// four write the first LSTM layer's input rows of this utterance's new hypotheses,
// gather_xh[pair, :] = bf16(h of the parent), which would otherwise take a kernel of its own between
// this one and the gate GEMM.
__device__ __forceinline__ unsigned rowfill_bf16(float f) {
    unsigned v = __float_as_uint(f);
    v += 0x7FFFu + ((v >> 16) & 1u);   // round to nearest, ties to even
    return v >> 16;
}

__global__ void __launch_bounds__(256)
k_rowfill(Dims d, int seg, const int *utt_off, AView A, RowView rv, int2 *nodes, int assign_nodes, int *host_counts,
          int seq, const float *gather_h, bf16_t *gather_xh) {
    __shared__ int s_pslot[TBS_MAX_BEAM];
    __shared__ int s_pair0, s_cnt;
    const int u = blockIdx.x;
    if (threadIdx.x < WAVE) rowfill_lists(d, seg, utt_off, A, rv, nodes, assign_nodes, host_counts, seq, u, threadIdx.x,
                                          gather_h != nullptr, s_pslot, &s_pair0, &s_cnt);
    if (gather_h == nullptr) return;   // (one wave launched)
    __syncthreads();
    const int cnt = s_cnt, pair0 = s_pair0, H4 = d.H >> 2, total = cnt * H4;
    for (int base = threadIdx.x; base < total; base += 256 * 4) {
        float4 v[4];
        int at[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int idx = min(base + k * 256, total - 1);
            const int h = idx / H4, i = idx - h * H4;
            v[k] = reinterpret_cast<const float4 *>(gather_h + (long)s_pslot[h] * d.H)[i];
            at[k] = (pair0 + h) * H4 + i;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (base + k * 256 < total)
                reinterpret_cast<uint2 *>(gather_xh)[at[k]] =
                    make_uint2(rowfill_bf16(v[k].x) | (rowfill_bf16(v[k].y) << 16),
                               rowfill_bf16(v[k].z) | (rowfill_bf16(v[k].w) << 16));
    }
}

hipError_t launch_rowfill(hipStream_t st, const Dims &d, int seg, const int *utt_off, AView A, RowView rv,
                          int2 *nodes, int assign_nodes, int *host_counts, int seq, const float *gather_h,
                          bf16_t *gather_xh) {
    if (gather_h && (d.H & 3)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_rowfill, dim3(d.U), dim3(gather_h ? 256 : WAVE), 0, st, d, seg, utt_off, A, rv, nodes,
                       assign_nodes, host_counts, seq, gather_h, gather_xh);
    return hipGetLastError();
}

// ------------------------------------------------------------------ select + merge
// Second half of the inner loop of Algorithm 1, one utterance per wave.  The
// utterance's B list, its A entries and its H*N candidates are staged in LDS
// with one round of parallel loads, all list work happens there, and B and the
// new A are written back once, so the kernel costs a handful of memory round
// trips instead of one per list operation.

__global__ void __launch_bounds__(WAVE)
k_select_merge(Dims d, int round, int drop, const float *logits, const float *row_lc,
               const float *dphi, const float *cand_score, const int *cand_tok, AView A, AView An, BView B,
               RowView rv, const int2 *nodes) {
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];   // B list of this utterance
    const int u = blockIdx.x;
    const int pair0 = rv.utt_pair0[u];
    const SelectFigs fg = select_figs(u, A, B, rv);
    SelectIn in;
    in.cand_score = cand_score + (long)pair0 * d.N;
    in.cand_tok = cand_tok + (long)pair0 * d.N;
    in.dphi = dphi + pair0;
    in.lc = row_lc + fg.urow0;
    in.slot_rows = 0;
    select_merge_utt(0, d, round, drop, u, (int)threadIdx.x, logits, in, fg, A, An, B, rv, nodes, s_dyn);
}

hipError_t launch_select_merge(hipStream_t st, const Dims &d, int round, int drop, const float *logits,
                               const float *row_lc, const float *dphi, const float *cand_score,
                               const int *cand_tok, AView A, AView An, BView B, RowView rv, const int2 *nodes) {
    const size_t shm = (size_t)d.BCAP * (sizeof(double) + sizeof(u64) + 3 * sizeof(int));
    // the longest B list the library accepts (2048 entries) needs 56 KB of dynamic LDS on top of
    // the kernel's static arrays: more than the default limit, so the limit is raised once
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_select_merge),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 2048 * (int)(sizeof(double) + sizeof(u64) + 3 * sizeof(int)));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(k_select_merge, dim3(d.U), dim3(WAVE), shm, st, d, round, drop, logits, row_lc, dphi,
                       cand_score, cand_tok, A, An, B, rv, nodes);
    return hipGetLastError();
}

// ------------------------------------------------------------------ results
__device__ void write_tokens(const int2 *nodes, int node, int len, int max_len, int *out) {
    // walk from the last token to the first
    int pos = len - 1;
    while (node > 0 && pos >= 0) {
        int2 nd = nodes[node];
        if (pos < max_len) out[pos] = nd.y;
        node = nd.x;
        --pos;
    }
}

// return ChooseNBest(B)   (Algorithm 1, last line)
// One wave per utterance writes every output entry of that utterance exactly once: ranks that
// exist get their score, length and tokens, everything else (ranks beyond the list, positions
// beyond a sequence) the neutral value, so the caller's buffers need no clearing beforehand.
__global__ void __launch_bounds__(WAVE)
k_finalize(Dims d, BView B, const int2 *nodes, int *res_count, int *res_len, double *res_logs,
           int *res_tok, int max_len) {
    __shared__ int s_len[TBS_MAX_BEAM];
    const int u = blockIdx.x, lane = threadIdx.x;
    const int nB = B.count[u];
    const double *bl = B.logs + (long)u * d.BCAP;
    if (lane < d.N) s_len[lane] = 0;
    __syncthreads();
    for (int i = lane; i < nB; i += WAVE) {
        double si = bl[i];
        int rank = 0;
        for (int j = 0; j < nB; ++j) {
            double sj = bl[j];
            rank += (sj > si) || (sj == si && j < i);
        }
        if (rank < d.N) {
            long o = (long)u * d.N + rank;
            int len = B.len[(long)u * d.BCAP + i];
            res_logs[o] = si;
            res_len[o] = len;
            s_len[rank] = len;
            write_tokens(nodes, B.node[(long)u * d.BCAP + i], len, max_len, res_tok + o * max_len);
        }
    }
    __syncthreads();
    const int cnt = nB < d.N ? nB : d.N;
    if (lane < d.N && lane >= cnt) {
        res_logs[(long)u * d.N + lane] = 0.0;
        res_len[(long)u * d.N + lane] = 0;
    }
    for (int idx = lane; idx < d.N * max_len; idx += WAVE) {
        const int r = idx / max_len, p = idx - r * max_len;
        if (p >= s_len[r]) res_tok[((long)u * d.N + r) * max_len + p] = -1;
    }
    if (lane == 0) res_count[u] = cnt;
}

hipError_t launch_finalize(hipStream_t st, const Dims &d, BView B, const int2 *nodes, int *res_count, int *res_len,
                           double *res_logs, int *res_tok, int max_len) {
    hipLaunchKernelGGL(k_finalize, dim3(d.U), dim3(WAVE), 0, st, d, B, nodes, res_count, res_len, res_logs, res_tok,
                       max_len);
    return hipGetLastError();
}

// Every entry of the four outputs is written exactly once (entries past the list and positions
// past a sequence get the neutral value), so the buffers need no clearing beforehand.
__global__ void __launch_bounds__(WAVE)
k_hyps_dump(Dims d, int group, AView A, BView B, const int2 *nodes, int cap, int max_len, int *tok,
            int *len, double *logs, int *count) {
    int u = blockIdx.x, lane = threadIdx.x;
    int n = group == 0 ? A.count[u] : B.count[u];
    int stride = group == 0 ? d.N : d.BCAP;
    if (n > cap) n = cap;
    for (int i = lane; i < cap; i += WAVE) {
        long s = (long)u * stride + i, o = (long)u * cap + i;
        if (i < n) {
            int ln = group == 0 ? A.len[s] : B.len[s];
            int nd = group == 0 ? A.node[s] : B.node[s];
            logs[o] = group == 0 ? A.logs[s] : B.logs[s];
            len[o] = ln;
            write_tokens(nodes, nd, ln, max_len, tok + o * max_len);
        } else {
            logs[o] = 0.0;
            len[o] = 0;
        }
    }
    for (int idx = lane; idx < cap * max_len; idx += WAVE) {
        const int i = idx / max_len, p = idx - i * max_len;
        int ln = 0;
        if (i < n) ln = group == 0 ? A.len[(long)u * stride + i] : B.len[(long)u * stride + i];
        if (p >= ln) tok[((long)u * cap + i) * max_len + p] = -1;
    }
    if (lane == 0) count[u] = n;
}

hipError_t launch_hyps_dump(hipStream_t st, const Dims &d, int group, AView A, BView B, const int2 *nodes, int cap,
                            int max_len, int *tok, int *len, double *logs, int *count) {
    hipLaunchKernelGGL(k_hyps_dump, dim3(d.U), dim3(WAVE), 0, st, d, group, A, B, nodes, cap, max_len, tok, len,
                       logs, count);
    return hipGetLastError();
}

// A_PRED view for tests: gather (scatter=0) or scatter (scatter=1) the projected
// predictor outputs of group A between the state pool and a dense [U,N,Dj] array.
__global__ void k_gather_pred(Dims d, AView A, float *pool_p, float *dense, int scatter) {
    int u = blockIdx.x / d.N, i = blockIdx.x % d.N;
    if (i >= A.count[u]) return;
    long a = (long)u * d.N + i;
    long slot = A.slot[a];
    for (int j = threadIdx.x; j < d.Dj; j += blockDim.x) {
        if (scatter) pool_p[slot * d.Dj + j] = dense[a * d.Dj + j];
        else dense[a * d.Dj + j] = pool_p[slot * d.Dj + j];
    }
}

hipError_t launch_gather_pred(hipStream_t st, const Dims &d, AView A, const float *pool_p, float *out, int scatter) {
    hipLaunchKernelGGL(k_gather_pred, dim3(d.U * d.N), dim3(256), 0, st, d, A, const_cast<float *>(pool_p), out,
                       scatter);
    return hipGetLastError();
}

// ------------------------------------------------------------------ test support
// After a test has written A_COUNT: give every entry of A a state slot of its
// own (arena 0, region 0) and the empty token sequence.
__global__ void k_debug_fill_a(Dims d, AView A) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= d.U * d.N) return;
    int u = idx / d.N, i = idx % d.N;
    A.slot[idx] = tbs_slot_id(u, 0, 0, i, d.R, d.N);
    A.pslot[idx] = A.slot[idx];
    A.node[idx] = 0;
    A.pnode[idx] = -1;
    A.token[idx] = -1;
    A.hash[idx] = 0ull;
    A.len[idx] = 0;
}

__global__ void k_set_sp(Dims d, int seg, const int *utt_T, RowView rv) {
    int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= d.U) return;
    int left = utt_T[u] - seg * d.S;
    rv.utt_sp[u] = left < 0 ? 0 : (left > d.S ? d.S : left);
    rv.utt_par[u] = 0;   // the arena k_debug_fill_a puts the hypotheses' states in
}

hipError_t launch_debug_fill_a(hipStream_t st, const Dims &d, AView A) {
    hipLaunchKernelGGL(k_debug_fill_a, dim3((d.U * d.N + 255) / 256), dim3(256), 0, st, d, A);
    return hipGetLastError();
}

hipError_t launch_set_sp(hipStream_t st, const Dims &d, int seg, const int *utt_T, RowView rv) {
    hipLaunchKernelGGL(k_set_sp, dim3((d.U + 255) / 256), dim3(256), 0, st, d, seg, utt_T, rv);
    return hipGetLastError();
}
