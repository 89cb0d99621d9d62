// Expansion scores of token-wise RNN-T beam search (Eq. 3-7) for every live
// hypothesis of a joiner call, and its N best non-blank expansions.
//
// One workgroup owns one (utterance, hypothesis) pair, i.e. the S' logit rows
// of that hypothesis.  Softmax probabilities are never formed: with row
// maximum m_t, row sum Z_t = sum_k exp(l[t,k]-m_t) and blank probability b_t,
// the blank products of Eq. 3 collapse into a forward variable
//     alpha_1 = d_old[1],  alpha_t = alpha_{t-1} b_{t-1} + d_old[t]
// (alpha_t = sum_{t1<=t} d_old[t1] Bl(t1,t)), so that
//     delta_blank   = alpha_S' b_S'                                  (Eq. 7; handed on as its logarithm)
//     d[k][t]       = alpha_t exp(l[t,k]-m_t) / Z_t                   (Eq. 4-5)
//     delta_nb[k]   = sum_t d[k][t] = sum_t exp(l[t,k] + lc_t)        (Eq. 6)
// with lc_t = log(alpha_t / Z_t) - m_t.  The [S+1,S+1] table, the [V,S] tensor
// d and the normalised J are never built; the logits are streamed from memory
// and each costs one exp and one add.
#include "tbs_internal.h"

#include "expand_device.h"

template <bool VEC4>
__global__ void __launch_bounds__(EXP_THREADS)
k_expand(Dims d, const float *__restrict__ logits, AView A, RowView rv, float *__restrict__ row_lc,
         float *__restrict__ dphi, float *__restrict__ cand_score, int *__restrict__ cand_tok,
         float *__restrict__ row_stats, float *__restrict__ delta_nb, const int *__restrict__ pairs_dev,
         int pair_base) {
    extern __shared__ float s_dnb[];  // [V]
    __shared__ float s_m[TBS_MAX_SEG], s_z[TBS_MAX_SEG], s_b[TBS_MAX_SEG], s_lc[TBS_MAX_SEG];
    __shared__ float s_rv[EXP_WAVES];
    __shared__ int s_rk[EXP_WAVES];
    const int pair = pair_base + blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (pairs_dev && pair >= *pairs_dev) return;   // (enqueued on an upper-bound grid, see k_expand_reg)
    const int u = rv.pair_u[pair], h = rv.pair_h[pair];
    const int row0 = rv.pair_row0[pair], sp = rv.pair_len[pair];
    const int V = d.V;
    const float *L = logits + (long)row0 * V;

    // ---- softmax statistics of each row: one wave per row, no barriers inside
    for (int t = wave; t < sp; t += EXP_WAVES) {
        const float *row = L + (long)t * V;
        float m = -INFINITY, z = 0.f;
        if (VEC4) {
            const float4 *r4 = reinterpret_cast<const float4 *>(row);
            for (int i = lane; i < V / 4; i += 64) {
                float4 x = r4[i];
                float mx = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
                float mn = fmaxf(m, mx);
                z = z * __expf(m - mn) + __expf(x.x - mn) + __expf(x.y - mn) + __expf(x.z - mn) + __expf(x.w - mn);
                m = mn;
            }
        } else {
            for (int i = lane; i < V; i += 64) {
                float x = row[i];
                float mn = fmaxf(m, x);
                z = z * __expf(m - mn) + __expf(x - mn);
                m = mn;
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            float m2 = __shfl_xor(m, off), z2 = __shfl_xor(z, off);
            ms_combine(m, z, m2, z2);
        }
        if (lane == 0) {
            s_m[t] = m;
            s_z[t] = z;
            s_b[t] = __expf(row[d.blank] - m) / z;
        }
    }
    __syncthreads();

    // ---- forward variable over the segment (Eq. 3 folded into a scan) and Eq. 7
    if (tid == 0) {
        const float *dold = A.dhat + ((long)u * d.N + h) * d.S;
        ScanAlpha al;
        al.start();
        for (int t = 0; t < sp; ++t) {
            al.step(t == 0 ? 0.f : s_b[t - 1], dold[t]);
            float lc = al.log_value() - __logf(s_z[t]) - s_m[t];   // log(alpha_t / Z_t) - m_t, no underflow
            s_lc[t] = lc;
            row_lc[row0 + t] = lc;
            if (row_stats) {
                row_stats[(long)(row0 + t) * 3 + 0] = s_m[t];
                row_stats[(long)(row0 + t) * 3 + 1] = s_z[t];
                row_stats[(long)(row0 + t) * 3 + 2] = s_b[t];
            }
        }
        dphi[pair] = al.log_times(s_b[sp - 1]);
    }
    __syncthreads();

    // ---- Eq. 4-6: delta_nb[k] = sum_t exp(l[t,k] + lc_t), streamed
    if (VEC4) {
        for (int i = tid; i < V / 4; i += EXP_THREADS) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int t = 0; t < sp; ++t) {
                float4 x = reinterpret_cast<const float4 *>(L + (long)t * V)[i];
                float lc = s_lc[t];
                acc.x += __expf(x.x + lc);
                acc.y += __expf(x.y + lc);
                acc.z += __expf(x.z + lc);
                acc.w += __expf(x.w + lc);
            }
            reinterpret_cast<float4 *>(s_dnb)[i] = acc;
        }
    } else {
        for (int k = tid; k < V; k += EXP_THREADS) {
            float acc = 0.f;
            for (int t = 0; t < sp; ++t) acc += __expf(L[(long)t * V + k] + s_lc[t]);
            s_dnb[k] = acc;
        }
    }
    __syncthreads();
    if (tid == 0) s_dnb[d.blank] = 0.f;  // blank is not a non-blank expansion
    __syncthreads();
    if (delta_nb)
        for (int k = tid; k < V; k += EXP_THREADS) delta_nb[(long)pair * V + k] = s_dnb[k];

    // ---- the N best expansions of this hypothesis: N rounds of workgroup arg-max
    for (int n = 0; n < d.N; ++n) {
        float bv = 0.f;  // only strictly positive scores are candidates
        int bk = 0x7fffffff;
        for (int k = tid; k < V; k += EXP_THREADS) {
            float v = s_dnb[k];
            if (v > bv) { bv = v; bk = k; }  // ascending k: the smallest token wins a tie
        }
        for (int off = 32; off > 0; off >>= 1) {
            float ov = __shfl_xor(bv, off);
            int ok = __shfl_xor(bk, off);
            if (ov > bv || (ov == bv && ok < bk)) { bv = ov; bk = ok; }
        }
        if (lane == 0) { s_rv[wave] = bv; s_rk[wave] = bk; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < EXP_WAVES; ++w)
                if (s_rv[w] > bv || (s_rv[w] == bv && s_rk[w] < bk)) { bv = s_rv[w]; bk = s_rk[w]; }
            if (bk != 0x7fffffff) {
                cand_score[(long)pair * d.N + n] = __logf(bv);
                cand_tok[(long)pair * d.N + n] = bk;
                s_dnb[bk] = -1.f;
            } else {
                cand_score[(long)pair * d.N + n] = -INFINITY;
                cand_tok[(long)pair * d.N + n] = -1;
            }
        }
        __syncthreads();
    }
}

template <int NV4, int SMAX>
__global__ void __launch_bounds__(EXP_THREADS, (NV4 * SMAX == 20 ? 5 : 1))   // 80 logits per thread: five waves per SIMD still fit
k_expand_reg(Dims d, const float *__restrict__ logits, AView A, RowView rv, float *__restrict__ row_lc,
             float *__restrict__ dphi, float *__restrict__ cand_score, int *__restrict__ cand_tok,
             float *__restrict__ row_stats, float *__restrict__ delta_nb, const int *__restrict__ pairs_dev,
             int pair_base) {
    __shared__ ExpandShared<SMAX, EXP_WAVES> sm;
    // Workgroup b runs on XCD b % 8.  The joiner GEMM before this kernel gave XCD x the x-th eighth
    // of the rows, in increasing order; here XCD x walks the pairs of the same eighth backwards, so
    // that what it reads first is what was written last (still in its L2 and in the memory-side
    // cache) and is read before this kernel's own traffic evicts it.  Measured: 196 -> 184 us at
    // 51200 rows x 4096.
    // (eighth x holds as many pairs as there are workgroups with b % 8 == x: every pair gets one)
    // (pairs_dev not null: the launch went out before the host knew the number of pairs; the grid is
    // an upper bound and the workgroups beyond the count in device memory leave)
    // (pair_base: the grid covers the pairs pair_base .. pair_base + gridDim.x - 1, one piece of a
    // large call, joined by a GEMM launch of its own over exactly these pairs' rows)
    int pair = blockIdx.x;
    if (pairs_dev) {
        if (pair >= *pairs_dev) return;
    } else {
        const int pairs = gridDim.x, q = pairs >> 3, r = pairs & 7, x = blockIdx.x & 7;
        const int first = x * q + min(x, r), count = q + (x < r);
        pair = first + count - 1 - (int)(blockIdx.x >> 3);
    }
    pair += pair_base;
    ExpandPair<SMAX> pi;
    expand_pair_info(pi, pair, d, A, rv, logits);
    float e[SMAX][NV4 * 4];
    expand_load<NV4, SMAX, EXP_THREADS>(e, logits, pi.row0, pi.sp, d.V, (int)threadIdx.x);
    expand_pair<NV4, SMAX, EXP_THREADS>(e, pi, sm, d, (int)threadIdx.x, true, row_lc + pi.row0, dphi + pi.pair,
                                        cand_score + (long)pi.pair * d.N, cand_tok + (long)pi.pair * d.N, row_stats,
                                        delta_nb);
}

template <int NV4, int SMAX>
static void expand_reg_launch(hipStream_t st, const Dims &d, int pairs, const float *logits, AView A, RowView rv,
                              float *row_lc, float *dphi, float *cand_score, int *cand_tok, float *row_stats,
                              float *delta_nb, const int *pairs_dev, int pair_base) {
    hipLaunchKernelGGL((k_expand_reg<NV4, SMAX>), dim3(pairs), dim3(EXP_THREADS), 0, st, d, logits, A, rv, row_lc, dphi,
                       cand_score, cand_tok, row_stats, delta_nb, pairs_dev, pair_base);
}

hipError_t launch_expand(hipStream_t st, const Dims &d, int pairs, const float *logits, AView A, RowView rv,
                         float *row_lc, float *dphi, float *cand_score, int *cand_tok, float *row_stats,
                         float *delta_nb, int force_generic, const int *pairs_dev, int pair_base) {
    if (pairs <= 0) return hipSuccess;
    if (pairs_dev && pair_base) return hipErrorInvalidValue;   // (a piece is launched with its size known)
    size_t shm = (size_t)d.V * sizeof(float);
    if (d.V % 4 == 0 && !force_generic) {
#define TBS_EXPAND_REG(NV4, SMAX)                                                                              \
    {                                                                                                          \
        expand_reg_launch<NV4, SMAX>(st, d, pairs, logits, A, rv, row_lc, dphi, cand_score, cand_tok, row_stats, \
                                     delta_nb, pairs_dev, pair_base);                                          \
        return hipGetLastError();                                                                              \
    }
        const int nv4 = (d.V / 4 + EXP_THREADS - 1) / EXP_THREADS;
        if (nv4 <= 1 && d.S <= 3) TBS_EXPAND_REG(1, 3)
        if (nv4 <= 1 && d.S <= 5) TBS_EXPAND_REG(1, 5)
        if (nv4 <= 1 && d.S <= 16) TBS_EXPAND_REG(1, 16)
        if (nv4 <= 2 && d.S <= 8) TBS_EXPAND_REG(2, 8)
        if (nv4 <= 4 && d.S <= 3) TBS_EXPAND_REG(4, 3)
        if (nv4 <= 4 && d.S <= 5) TBS_EXPAND_REG(4, 5)
#undef TBS_EXPAND_REG
    }
    if (d.V % 4 == 0)
        hipLaunchKernelGGL(k_expand<true>, dim3(pairs), dim3(EXP_THREADS), shm, st, d, logits, A, rv, row_lc, dphi,
                           cand_score, cand_tok, row_stats, delta_nb, pairs_dev, pair_base);
    else
        hipLaunchKernelGGL(k_expand<false>, dim3(pairs), dim3(EXP_THREADS), shm, st, d, logits, A, rv, row_lc, dphi,
                           cand_score, cand_tok, row_stats, delta_nb, pairs_dev, pair_base);
    return hipGetLastError();
}
