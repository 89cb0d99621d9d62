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

#define WAVE 64

__device__ __forceinline__ double log_add(double a, double b) {
    double mx = a > b ? a : b, mn = a > b ? b : a;
    if (isinf(mx)) return mx;
    return mx + log1p(exp(mn - mx));
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
        if (u == 0) {
            nodes[0] = make_int2(-1, -1);
            rv.counts[TBS_CNT_PAIRS] = 0;
            rv.counts[TBS_CNT_ROWS] = 0;
            rv.counts[TBS_CNT_NODES] = 1;
            rv.counts[TBS_CNT_ERR] = 0;
            rv.counts[TBS_CNT_UTTS] = 0;
            rv.counts[TBS_CNT_FRAMES] = 0;
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
__global__ void k_segment_begin(Dims d, int seg, int parity, const int *utt_T, BView B, AView A, RowView rv) {
    int u = blockIdx.x, lane = threadIdx.x;
    int left = utt_T[u] - seg * d.S;
    int sp = left < 0 ? 0 : (left > d.S ? d.S : left);
    if (lane == 0) rv.utt_sp[u] = sp;
    if (sp == 0) {  // finished (or empty) utterance: B keeps the final list
        if (lane == 0) A.count[u] = 0;
        return;
    }
    int nB = B.count[u];
    const double *bl = B.logs + (long)u * d.BCAP;
    for (int i = lane; i < nB; i += WAVE) {
        double si = bl[i];
        int rank = 0;
        for (int j = 0; j < nB; ++j) {
            double sj = bl[j];
            rank += (sj > si) || (sj == si && j < i);
        }
        if (rank < d.N) {
            long a = (long)u * d.N + rank, b = (long)u * d.BCAP + i;
            A.logs[a] = si;
            A.node[a] = B.node[b];
            A.hash[a] = B.hash[b];
            A.len[a] = B.len[b];
            A.pslot[a] = B.slot[b];
            A.slot[a] = tbs_slot_id(u, parity, 0, rank, d.R, d.N);
            A.pnode[a] = -1;
            A.token[a] = -1;
            float *dh = A.dhat + a * d.S;
            dh[0] = 1.f;
            for (int t = 1; t < d.S; ++t) dh[t] = 0.f;
        }
    }
    __syncthreads();
    if (lane == 0) {
        A.count[u] = nB < d.N ? nB : d.N;
        B.count[u] = 0;
    }
}

hipError_t launch_segment_begin(hipStream_t st, const Dims &d, int seg, int parity, const int *utt_T, BView B,
                                AView A, RowView rv) {
    hipLaunchKernelGGL(k_segment_begin, dim3(d.U), dim3(WAVE), 0, st, d, seg, parity, utt_T, B, A, rv);
    return hipGetLastError();
}

// Survivors move their predictor state into this segment's arena (slot r=0).
__global__ void k_state_copy(Dims d, AView A, RowView rv, float *pool_p, float *pool_h, float *pool_c,
                             long pool_rows) {
    int u = blockIdx.x / d.N, i = blockIdx.x % d.N;
    if (rv.utt_sp[u] == 0 || i >= A.count[u]) return;
    long a = (long)u * d.N + i;
    long src = A.pslot[a], dst = A.slot[a];
    for (int j = threadIdx.x; j < d.Dj; j += blockDim.x) pool_p[dst * d.Dj + j] = pool_p[src * d.Dj + j];
    for (int l = 0; l < d.L; ++l)
        for (int j = threadIdx.x; j < d.H; j += blockDim.x) {
            pool_h[((long)l * pool_rows + dst) * d.H + j] = pool_h[((long)l * pool_rows + src) * d.H + j];
            pool_c[((long)l * pool_rows + dst) * d.H + j] = pool_c[((long)l * pool_rows + src) * d.H + j];
        }
}

hipError_t launch_state_copy(hipStream_t st, const Dims &d, AView A, RowView rv, float *pool_p, float *pool_h,
                             float *pool_c, long pool_rows) {
    hipLaunchKernelGGL(k_state_copy, dim3(d.U * d.N), dim3(256), 0, st, d, A, rv, pool_p, pool_h, pool_c,
                       pool_rows);
    return hipGetLastError();
}

// ------------------------------------------------------------------ row list
// Compacts the live (utterance, hypothesis) pairs and their (pair, frame) rows
// for one joiner call, gives new hypotheses their trie nodes, and publishes the
// counts to the host.  One workgroup; U is at most a few thousand.
__global__ void k_rowlist(Dims d, int seg, const int *utt_T, const int *utt_off, AView A, RowView rv, int2 *nodes,
                          int assign_nodes, int *host_counts) {
    __shared__ int s_pairs[1024], s_rows[1024];
    __shared__ int s_carry[4];
    int tid = threadIdx.x;
    if (tid == 0) { s_carry[0] = 0; s_carry[1] = 0; s_carry[2] = 0; s_carry[3] = 0; }
    __syncthreads();
    int node_base = rv.counts[TBS_CNT_NODES];
    for (int base = 0; base < d.U; base += 1024) {
        int u = base + tid;
        int cnt = 0, sp = 0;
        if (u < d.U) {
            sp = rv.utt_sp[u];
            cnt = sp > 0 ? A.count[u] : 0;
        }
        s_pairs[tid] = cnt;
        s_rows[tid] = cnt * sp;
        __syncthreads();
        // inclusive Hillis-Steele scan over the chunk
        for (int off = 1; off < 1024; off <<= 1) {
            int vp = 0, vr = 0;
            if (tid >= off) { vp = s_pairs[tid - off]; vr = s_rows[tid - off]; }
            __syncthreads();
            s_pairs[tid] += vp;
            s_rows[tid] += vr;
            __syncthreads();
        }
        int pair0 = s_carry[0] + s_pairs[tid] - cnt;
        int row0 = s_carry[1] + s_rows[tid] - cnt * sp;
        if (u < d.U) {
            rv.utt_pair0[u] = pair0;
            int t0 = seg * d.S;
            for (int h = 0; h < cnt; ++h) {
                int j = pair0 + h;
                long a = (long)u * d.N + h;
                rv.pair_u[j] = u;
                rv.pair_h[j] = h;
                rv.pair_row0[j] = row0 + h * sp;
                rv.pair_len[j] = sp;
                int slot = A.slot[a];
                for (int t = 0; t < sp; ++t) {
                    rv.row_enc[row0 + h * sp + t] = utt_off[u] + t0 + t;
                    rv.row_slot[row0 + h * sp + t] = slot;
                }
                if (assign_nodes) {
                    int node = node_base + j;
                    if (node < d.max_nodes) {
                        nodes[node] = make_int2(A.pnode[a], A.token[a]);
                        A.node[a] = node;
                    } else {
                        A.node[a] = 0;
                    }
                }
            }
        }
        __syncthreads();
        if (tid == 1023) {
            s_carry[0] += s_pairs[1023];
            s_carry[1] += s_rows[1023];
        }
        if (cnt > 0) { atomicAdd(&s_carry[2], 1); atomicAdd(&s_carry[3], sp); }
        __syncthreads();
    }
    if (tid == 0) {
        int pairs = s_carry[0], rows = s_carry[1];
        int err = rv.counts[TBS_CNT_ERR];
        int nodes_used = node_base;
        if (assign_nodes) {
            nodes_used = node_base + pairs;
            if (nodes_used > d.max_nodes) { err |= TBS_ERRF_NODES; nodes_used = d.max_nodes; }
        }
        rv.counts[TBS_CNT_PAIRS] = pairs;
        rv.counts[TBS_CNT_ROWS] = rows;
        rv.counts[TBS_CNT_NODES] = nodes_used;
        rv.counts[TBS_CNT_ERR] = err;
        rv.counts[TBS_CNT_UTTS] = s_carry[2];
        rv.counts[TBS_CNT_FRAMES] = s_carry[3];
        if (host_counts) {  // pinned, device-mapped host memory: the host reads it after a stream sync
            host_counts[TBS_CNT_PAIRS] = pairs;
            host_counts[TBS_CNT_ROWS] = rows;
            host_counts[TBS_CNT_NODES] = nodes_used;
            host_counts[TBS_CNT_ERR] = err;
            host_counts[TBS_CNT_UTTS] = s_carry[2];
            host_counts[TBS_CNT_FRAMES] = s_carry[3];
            __threadfence_system();
        }
    }
}

hipError_t launch_rowlist(hipStream_t st, const Dims &d, int seg, const int *utt_T, const int *utt_off, AView A,
                          RowView rv, int2 *nodes, int assign_nodes, int *host_counts) {
    hipLaunchKernelGGL(k_rowlist, dim3(1), dim3(1024), 0, st, d, seg, utt_T, utt_off, A, rv, nodes, assign_nodes,
                       host_counts);
    return hipGetLastError();
}

// ------------------------------------------------------------------ select + merge
// Second half of the inner loop of Algorithm 1 for one utterance per wave.
#define CAND_MAX (TBS_MAX_BEAM * TBS_MAX_BEAM)

__global__ void __launch_bounds__(WAVE)
k_select_merge(Dims d, int parity, int round, int drop, const float *logits, const float *row_lc,
               const float *dphi, const float *cand_score, const int *cand_tok, AView A, AView An, BView B,
               RowView rv, const int2 *nodes) {
    __shared__ double s_key[CAND_MAX];
    __shared__ int s_sel[TBS_MAX_BEAM];      // candidate index by rank
    __shared__ int s_keep[TBS_MAX_BEAM];
    __shared__ int s_found;
    __shared__ double s_thr;
    const int u = blockIdx.x, lane = threadIdx.x;
    const int N = d.N;
    const int H = rv.utt_sp[u] > 0 ? A.count[u] : 0;
    if (H == 0) {
        if (lane == 0) An.count[u] = 0;
        return;
    }
    const int pair0 = rv.utt_pair0[u];
    double *bl = B.logs + (long)u * d.BCAP;
    int *bnode = B.node + (long)u * d.BCAP;
    u64 *bhash = B.hash + (long)u * d.BCAP;
    int *blen = B.len + (long)u * d.BCAP;
    int *bslot = B.slot + (long)u * d.BCAP;
    int nB = B.count[u];

    // --- AddAndMerge of every blank expansion, in hypothesis order
    for (int h = 0; h < H; ++h) {
        long a = (long)u * N + h;
        double key = A.logs[a] + log((double)dphi[pair0 + h]);
        u64 hs = A.hash[a];
        int ln = A.len[a], nd = A.node[a];
        if (lane == 0) s_found = 0x7fffffff;
        __syncthreads();
        for (int base = 0; base < nB; base += WAVE) {
            int i = base + lane;
            bool hit = false;
            if (i < nB && bhash[i] == hs && blen[i] == ln) hit = same_sequence(nodes, bnode[i], nd);
            if (hit) atomicMin(&s_found, i);  // at most one entry can match; min keeps it deterministic
        }
        __syncthreads();
        int f = s_found == 0x7fffffff ? -1 : s_found;
        if (lane == 0) {
            if (f >= 0) {
                bl[f] = log_add(bl[f], key);
            } else if (nB < d.BCAP) {
                bl[nB] = key;
                bnode[nB] = nd;
                bhash[nB] = hs;
                blen[nB] = ln;
                bslot[nB] = A.slot[a];
            } else {
                atomicOr(&rv.counts[TBS_CNT_ERR], TBS_ERRF_BCAP);
            }
        }
        if (f < 0 && nB < d.BCAP) ++nB;
        __syncthreads();
    }
    if (lane == 0) B.count[u] = nB;

    // --- threshold = ChooseNthScore(B, N), only defined when B holds N entries
    const bool have_thr = nB >= N;
    if (have_thr) {
        for (int i = lane; i < nB; i += WAVE) {
            double si = bl[i];
            int rank = 0;
            for (int j = 0; j < nB; ++j) {
                double sj = bl[j];
                rank += (sj > si) || (sj == si && j < i);
            }
            if (rank == N - 1) s_thr = si;
        }
    }
    __syncthreads();
    const double thr = have_thr ? s_thr : 0.0;

    // --- ChooseNBestExpansions: joint top-N over the H*N per-hypothesis candidates
    const int nc = H * N;
    for (int c = lane; c < nc; c += WAVE) {
        int h = c / N;
        int tok = cand_tok[(long)(pair0 + h) * N + (c % N)];
        double key = -INFINITY;
        if (tok >= 0) key = A.logs[(long)u * N + h] + (double)cand_score[(long)(pair0 + h) * N + (c % N)];
        s_key[c] = tok >= 0 ? key : nan("");
    }
    if (lane < N) { s_sel[lane] = -1; s_keep[lane] = 0; }
    __syncthreads();
    for (int c = lane; c < nc; c += WAVE) {
        double kc = s_key[c];
        if (kc != kc) continue;  // no candidate in this place
        int hc = c / N, tc = cand_tok[(long)(pair0 + hc) * N + (c % N)];
        int rank = 0;
        for (int j = 0; j < nc; ++j) {
            double kj = s_key[j];
            if (kj != kj || j == c) continue;
            int hj = j / N;
            bool better = kj > kc;
            if (kj == kc) {
                int tj = cand_tok[(long)(pair0 + hj) * N + (j % N)];
                better = (hj < hc) || (hj == hc && tj < tc);
            }
            rank += better;
        }
        if (rank < N) s_sel[rank] = c;
    }
    __syncthreads();
    // --- threshold test, in rank order: keep iff |B| < N or score > threshold (strict)
    if (lane < N) {
        int c = s_sel[lane];
        if (c >= 0) s_keep[lane] = (!have_thr) || (s_key[c] > thr);
    }
    __syncthreads();
    if (drop) {
        if (lane == 0) An.count[u] = 0;
        return;
    }
    int pos = 0, total = 0;
    for (int r = 0; r < N; ++r) {
        int k = s_keep[r];
        if (r < lane) pos += k;
        total += k;
    }
    if (lane == 0) An.count[u] = total;
    if (lane < N && s_keep[lane]) {
        int c = s_sel[lane];
        int h = c / N;
        int tok = cand_tok[(long)(pair0 + h) * N + (c % N)];
        long a = (long)u * N + h, an = (long)u * N + pos;
        An.logs[an] = s_key[c];
        An.pnode[an] = A.node[a];
        An.node[an] = -1;
        An.token[an] = tok;
        An.hash[an] = hash_append(A.hash[a], tok);
        An.len[an] = A.len[a] + 1;
        An.pslot[an] = A.slot[a];
        An.slot[an] = tbs_slot_id(u, parity, round, pos, d.R, N);
        // d of the new hypothesis (Eq. 5 for the chosen token), normalised by its sum (Eq. 6)
        int row0 = rv.pair_row0[pair0 + h], sp = rv.pair_len[pair0 + h];
        float *dh = An.dhat + an * d.S;
        float sum = 0.f;
        for (int t = 0; t < sp; ++t) {
            float x = __expf(logits[(long)(row0 + t) * d.V + tok] + row_lc[row0 + t]);
            dh[t] = x;
            sum += x;
        }
        float inv = 1.f / sum;
        for (int t = 0; t < sp; ++t) dh[t] *= inv;
        for (int t = sp; t < d.S; ++t) dh[t] = 0.f;
    }
}

hipError_t launch_select_merge(hipStream_t st, const Dims &d, int parity, int round, int drop, const float *logits,
                               const float *row_lc, const float *dphi, const float *cand_score,
                               const int *cand_tok, AView A, AView An, BView B, RowView rv, const int2 *nodes) {
    hipLaunchKernelGGL(k_select_merge, dim3(d.U), dim3(WAVE), 0, st, d, parity, round, drop, logits, row_lc, dphi,
                       cand_score, cand_tok, A, An, B, rv, nodes);
    return hipGetLastError();
}

// ------------------------------------------------------------------ results
__device__ void write_tokens(const int2 *nodes, int node, int len, int max_len, int *out, int *ovf) {
    // walk from the last token to the first
    int pos = len - 1;
    while (node > 0 && pos >= 0) {
        int2 nd = nodes[node];
        if (pos < max_len) out[pos] = nd.y;
        node = nd.x;
        --pos;
    }
    if (len > max_len) atomicOr(ovf, 1);
}

// return ChooseNBest(B)   (Algorithm 1, last line)
__global__ void k_finalize(Dims d, BView B, const int2 *nodes, int *res_count, int *res_len, double *res_logs,
                           int *res_tok, int max_len, int *ovf) {
    int u = blockIdx.x, lane = threadIdx.x;
    int nB = B.count[u];
    const double *bl = B.logs + (long)u * d.BCAP;
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
            write_tokens(nodes, B.node[(long)u * d.BCAP + i], len, max_len, res_tok + o * max_len, ovf);
        }
    }
    if (lane == 0) res_count[u] = nB < d.N ? nB : d.N;
}

hipError_t launch_finalize(hipStream_t st, const Dims &d, BView B, const int2 *nodes, int *res_count, int *res_len,
                           double *res_logs, int *res_tok, int max_len, int *ovf) {
    hipLaunchKernelGGL(k_finalize, dim3(d.U), dim3(WAVE), 0, st, d, B, nodes, res_count, res_len, res_logs, res_tok,
                       max_len, ovf);
    return hipGetLastError();
}

__global__ void k_hyps_dump(Dims d, int group, AView A, BView B, const int2 *nodes, int cap, int max_len, int *tok,
                            int *len, double *logs, int *count) {
    int u = blockIdx.x, lane = threadIdx.x;
    int n = group == 0 ? A.count[u] : B.count[u];
    int stride = group == 0 ? d.N : d.BCAP;
    if (n > cap) n = cap;
    int dummy = 0;
    for (int i = lane; i < n; i += WAVE) {
        long s = (long)u * stride + i, o = (long)u * cap + i;
        int ln = group == 0 ? A.len[s] : B.len[s];
        int nd = group == 0 ? A.node[s] : B.node[s];
        logs[o] = group == 0 ? A.logs[s] : B.logs[s];
        len[o] = ln;
        write_tokens(nodes, nd, ln, max_len, tok + o * max_len, &dummy);
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
}

hipError_t launch_debug_fill_a(hipStream_t st, const Dims &d, AView A) {
    hipLaunchKernelGGL(k_debug_fill_a, dim3((d.U * d.N + 255) / 256), dim3(256), 0, st, d, A);
    return hipGetLastError();
}

hipError_t launch_set_sp(hipStream_t st, const Dims &d, int seg, const int *utt_T, RowView rv) {
    hipLaunchKernelGGL(k_set_sp, dim3((d.U + 255) / 256), dim3(256), 0, st, d, seg, utt_T, rv);
    return hipGetLastError();
}
