// Expansion scores of token-wise RNN-T beam search (Eq. 3-7) for every live
// hypothesis of a joiner call, and its N best non-blank expansions.
//
// One workgroup owns one (utterance, hypothesis) pair, i.e. the S' logit rows
// of that hypothesis.  Softmax probabilities are never formed: with row
// maximum m_t, row sum Z_t = sum_k exp(l[t,k]-m_t) and blank probability b_t,
// the blank products of Eq. 3 collapse into a forward variable
//     alpha_1 = d_old[1],  alpha_t = alpha_{t-1} b_{t-1} + d_old[t]
// (alpha_t = sum_{t1<=t} d_old[t1] Bl(t1,t)), so that
//     delta_blank   = alpha_S' b_S'                                  (Eq. 7)
//     d[k][t]       = alpha_t exp(l[t,k]-m_t) / Z_t                   (Eq. 4-5)
//     delta_nb[k]   = sum_t d[k][t] = sum_t exp(l[t,k] + lc_t)        (Eq. 6)
// with lc_t = log(alpha_t / Z_t) - m_t.  The [S+1,S+1] table, the [V,S] tensor
// d and the normalised J are never built; the logits are streamed from memory
// and each costs one exp and one add.
#include "tbs_internal.h"

#define EXP_THREADS 256
#define EXP_WAVES (EXP_THREADS / 64)
#define EXP_CAND_CAP 64   // candidates one wave may hand to the merge (>= TBS_MAX_BEAM)

__device__ __forceinline__ void ms_combine(float &m, float &z, float m2, float z2) {
    float mn = fmaxf(m, m2);
    // exp(-inf - finite) = 0; guard the -inf - -inf case of two empty parts
    float a = (m == -INFINITY) ? 0.f : z * __expf(m - mn);
    float b = (m2 == -INFINITY) ? 0.f : z2 * __expf(m2 - mn);
    m = mn;
    z = a + b;
}

// ---- wave-wide reductions without LDS traffic: four DPP steps make every lane of a 16-lane row
// hold the row's result, four scalar lane reads combine the rows.  The result is uniform.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
#define DPP_QUAD_SWAP1 0xB1   // quad_perm [1,0,3,2]
#define DPP_QUAD_SWAP2 0x4E   // quad_perm [2,3,0,1]
#define DPP_HALF_MIRROR 0x141
#define DPP_MIRROR 0x140
__device__ __forceinline__ float lane_f(float v, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f<DPP_QUAD_SWAP1>(v));
    v = fmaxf(v, dpp_f<DPP_QUAD_SWAP2>(v));
    v = fmaxf(v, dpp_f<DPP_HALF_MIRROR>(v));
    v = fmaxf(v, dpp_f<DPP_MIRROR>(v));
    return fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f<DPP_QUAD_SWAP1>(v);
    v += dpp_f<DPP_QUAD_SWAP2>(v);
    v += dpp_f<DPP_HALF_MIRROR>(v);
    v += dpp_f<DPP_MIRROR>(v);
    return (lane_f(v, 0) + lane_f(v, 16)) + (lane_f(v, 32) + lane_f(v, 48));
}
__device__ __forceinline__ int wave_min_int(int v) {
    v = min(v, dpp_i<DPP_QUAD_SWAP1>(v));
    v = min(v, dpp_i<DPP_QUAD_SWAP2>(v));
    v = min(v, dpp_i<DPP_HALF_MIRROR>(v));
    v = min(v, dpp_i<DPP_MIRROR>(v));
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
// largest value of the wave and, among the lanes that hold it, the smallest key
__device__ __forceinline__ void wave_argmax(float &bv, int &bk) {
    const float wm = wave_max(bv);
    bk = wave_min_int(bv == wm ? bk : 0x7fffffff);
    bv = wm;
}

template <bool VEC4>
__global__ void __launch_bounds__(EXP_THREADS)
k_expand(Dims d, const float *__restrict__ logits, AView A, RowView rv, float *__restrict__ row_lc,
         float *__restrict__ dphi, float *__restrict__ cand_score, int *__restrict__ cand_tok,
         float *__restrict__ row_stats, float *__restrict__ delta_nb) {
    extern __shared__ float s_dnb[];  // [V]
    __shared__ float s_m[TBS_MAX_SEG], s_z[TBS_MAX_SEG], s_b[TBS_MAX_SEG], s_lc[TBS_MAX_SEG];
    __shared__ float s_rv[EXP_WAVES];
    __shared__ int s_rk[EXP_WAVES];
    const int pair = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
        float alpha = 0.f;
        for (int t = 0; t < sp; ++t) {
            alpha = (t == 0 ? 0.f : alpha * s_b[t - 1]) + dold[t];
            float c = alpha / s_z[t];
            float lc = c > 0.f ? __logf(c) - s_m[t] : -INFINITY;
            s_lc[t] = lc;
            row_lc[row0 + t] = lc;
            if (row_stats) {
                row_stats[(long)(row0 + t) * 3 + 0] = s_m[t];
                row_stats[(long)(row0 + t) * 3 + 1] = s_z[t];
                row_stats[(long)(row0 + t) * 3 + 2] = s_b[t];
            }
        }
        dphi[pair] = alpha * s_b[sp - 1];
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

// ------------------------------------------------------------------ register-resident variant
// When the S' x V logits of one hypothesis fit in the registers of one workgroup
// (V <= 1024 NV4 columns, S' <= SMAX), every logit is read from memory exactly
// once and exponentiated exactly once: the row maxima m_t are reduced across the
// workgroup first, each thread then keeps e = exp(l - m_t) of its own columns,
// the row sums Z_t follow from one more reduction, and the streaming sum of
// Eq. 4-6 becomes delta_nb[k] = sum_t c_t e[t][k] from registers.  The N best
// are then taken per wave from registers and merged by the first wave.
template <int NV4, int SMAX>
__global__ void __launch_bounds__(EXP_THREADS)
k_expand_reg(Dims d, const float *__restrict__ logits, AView A, RowView rv, float *__restrict__ row_lc,
             float *__restrict__ dphi, float *__restrict__ cand_score, int *__restrict__ cand_tok,
             float *__restrict__ row_stats, float *__restrict__ delta_nb) {
    constexpr int NC = NV4 * 4;  // columns per thread
    __shared__ float s_pm[EXP_WAVES][SMAX], s_pz[EXP_WAVES][SMAX];
    __shared__ float s_blank[SMAX];
    __shared__ float s_cv[EXP_WAVES][EXP_CAND_CAP];
    __shared__ int s_ck[EXP_WAVES][EXP_CAND_CAP];
    __shared__ int s_cn[EXP_WAVES];
    const int pair = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = rv.pair_u[pair], h = rv.pair_h[pair];
    const int row0 = rv.pair_row0[pair], sp = rv.pair_len[pair];
    const int V = d.V, V4 = V >> 2;
    const float4 *L4 = reinterpret_cast<const float4 *>(logits + (long)row0 * V);

    // ---- one pass over memory: this thread's columns of every row
    float e[SMAX][NC];
    float mrow[SMAX];
#pragma unroll
    for (int t = 0; t < SMAX; ++t) {
        mrow[t] = -INFINITY;
        if (t < sp) {
#pragma unroll
            for (int q = 0; q < NV4; ++q) {
                const int i4 = tid + EXP_THREADS * q;
                float4 x = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                if (i4 < V4) x = L4[(long)t * V4 + i4];
                e[t][4 * q + 0] = x.x; e[t][4 * q + 1] = x.y; e[t][4 * q + 2] = x.z; e[t][4 * q + 3] = x.w;
                mrow[t] = fmaxf(mrow[t], fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w)));
            }
        } else {
#pragma unroll
            for (int c = 0; c < NC; ++c) e[t][c] = -INFINITY;
        }
    }
    // ---- row maxima across the workgroup (waves by shuffles, then through LDS)
#pragma unroll
    for (int t = 0; t < SMAX; ++t) {
        const float m = wave_max(mrow[t]);
        if (lane == 0) s_pm[wave][t] = m;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < SMAX; ++t) {
        float m = s_pm[0][t];
#pragma unroll
        for (int w = 1; w < EXP_WAVES; ++w) m = fmaxf(m, s_pm[w][t]);
        mrow[t] = t < sp ? m : 0.f;
    }
    // ---- e = exp(l - m_t), once per logit; row sums across the workgroup; the owner of the blank
    // column publishes its exponentials
    {
        const int bq = (d.blank >> 2) / EXP_THREADS, bt = (d.blank >> 2) % EXP_THREADS, bc = d.blank & 3;
#pragma unroll
        for (int t = 0; t < SMAX; ++t) {
            const float nm = -mrow[t] * 1.44269504088896341f;
            float z = 0.f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                e[t][c] = __builtin_amdgcn_exp2f(fmaf(e[t][c], 1.44269504088896341f, nm));
                z += e[t][c];
            }
            z = wave_sum(z);
            if (lane == 0) s_pz[wave][t] = z;
            if (tid == bt) {
#pragma unroll
                for (int q = 0; q < NV4; ++q)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (q == bq && c == bc) s_blank[t] = e[t][4 * q + c];
            }
        }
    }
    __syncthreads();
    // ---- every thread: row sums, forward variable (Eq. 3 as a scan), Eq. 7, the row coefficients
    float cf[SMAX];
    {
        const float *dold = A.dhat + ((long)u * d.N + h) * d.S;
        float alpha = 0.f, bprev = 0.f;
#pragma unroll
        for (int t = 0; t < SMAX; ++t) {
            cf[t] = 0.f;
            if (t < sp) {
                float z = s_pz[0][t];
#pragma unroll
                for (int w = 1; w < EXP_WAVES; ++w) z += s_pz[w][t];
                const float b = s_blank[t] / z;
                alpha = (t == 0 ? 0.f : alpha * bprev) + dold[t];
                bprev = b;
                const float c = alpha / z;
                cf[t] = c;
                if (tid == 0) {
                    row_lc[row0 + t] = c > 0.f ? __logf(c) - mrow[t] : -INFINITY;
                    if (row_stats) {
                        row_stats[(long)(row0 + t) * 3 + 0] = mrow[t];
                        row_stats[(long)(row0 + t) * 3 + 1] = z;
                        row_stats[(long)(row0 + t) * 3 + 2] = b;
                    }
                    if (t == sp - 1) dphi[pair] = alpha * b;
                }
            }
        }
    }
    // ---- Eq. 4-6 from registers
    float v[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        float acc = 0.f;
#pragma unroll
        for (int t = 0; t < SMAX; ++t) acc += cf[t] * e[t][c];
        v[c] = acc;
    }
    // blank is not a non-blank expansion; columns past V do not exist
#pragma unroll
    for (int q = 0; q < NV4; ++q)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int col = 4 * (tid + EXP_THREADS * q) + c;
            if (col == d.blank || col >= V) v[4 * q + c] = 0.f;
        }
    if (delta_nb) {
#pragma unroll
        for (int q = 0; q < NV4; ++q) {
            const int i4 = tid + EXP_THREADS * q;
            if (i4 < V4)
                reinterpret_cast<float4 *>(delta_nb + (long)pair * V)[i4] =
                    make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
        }
    }
    // ---- candidates of this wave.  tau = the N-th largest of the 64 per-thread maxima is a lower
    // bound of the wave's N-th largest score, so every score >= tau is a candidate (ties included)
    // and usually only a few more than N qualify.  tau comes from N rounds of wave maximum over the
    // thread maxima (one lane retires per round); candidates are compacted with ballots.
    float tau = 0.f;
    {
        float lm = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) lm = fmaxf(lm, v[c]);
        for (int n = 0; n < d.N; ++n) {
            tau = wave_max(lm);
            if (!(tau > 0.f)) break;   // fewer than N positive maxima: every positive score qualifies
            const u64 holders = __ballot(lm == tau);
            if (lane == __ffsll((long long)holders) - 1) lm = -1.f;
        }
    }
    int total = 0;
    {
        const u64 below = (1ull << lane) - 1ull;
#pragma unroll
        for (int q = 0; q < NV4; ++q)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float x = v[4 * q + c];
                const bool take = x > 0.f && x >= tau;
                const u64 m = __ballot(take);
                const int pos = total + __popcll(m & below);
                if (take && pos < EXP_CAND_CAP) {
                    s_cv[wave][pos] = x;
                    s_ck[wave][pos] = 4 * (tid + EXP_THREADS * q) + c;
                }
                total += __popcll(m);
            }
    }
    if (total <= EXP_CAND_CAP) {
        if (lane == 0) s_cn[wave] = total;
    } else {
        // many equal scores: take exactly the N best by N rounds of wave arg-max
        for (int n = 0; n < d.N; ++n) {
            float bv = 0.f;
            int bk = 0x7fffffff;
#pragma unroll
            for (int q = 0; q < NV4; ++q)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float x = v[4 * q + c];
                    if (x > bv) { bv = x; bk = 4 * (tid + EXP_THREADS * q) + c; }   // ascending columns
                }
            wave_argmax(bv, bk);
            if (lane == 0) { s_cv[wave][n] = bv; s_ck[wave][n] = bk; }
#pragma unroll
            for (int q = 0; q < NV4; ++q)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (4 * (tid + EXP_THREADS * q) + c == bk) v[4 * q + c] = -1.f;
        }
        if (lane == 0) s_cn[wave] = d.N;
    }
    __syncthreads();
    // ---- merge the waves' candidate lists (first wave): N rounds of arg-max, larger score first,
    // smaller token on equal scores
    if (wave == 0) {
        float cv[EXP_WAVES];
        int ck[EXP_WAVES];
        int base = 0;
#pragma unroll
        for (int i = 0; i < EXP_WAVES; ++i) { cv[i] = -1.f; ck[i] = 0x7fffffff; }
#pragma unroll
        for (int w = 0; w < EXP_WAVES; ++w) {
            const int n_w = s_cn[w];
            // entry e of list w has global index base+e; lane takes indices lane, lane+64, ...
#pragma unroll
            for (int i = 0; i < EXP_WAVES; ++i) {
                const int e = lane + 64 * i - base;
                if (e >= 0 && e < n_w) { cv[i] = s_cv[w][e]; ck[i] = s_ck[w][e]; }
            }
            base += n_w;
        }
        for (int n = 0; n < d.N; ++n) {
            float bv = -1.f;
            int bk = 0x7fffffff;
#pragma unroll
            for (int i = 0; i < EXP_WAVES; ++i)
                if (cv[i] > bv || (cv[i] == bv && ck[i] < bk)) { bv = cv[i]; bk = ck[i]; }
            wave_argmax(bv, bk);
            if (lane == 0) {
                const bool ok = bv > 0.f && bk != 0x7fffffff;
                cand_score[(long)pair * d.N + n] = ok ? __logf(bv) : -INFINITY;
                cand_tok[(long)pair * d.N + n] = ok ? bk : -1;
            }
#pragma unroll
            for (int i = 0; i < EXP_WAVES; ++i)
                if (ck[i] == bk) { cv[i] = -1.f; ck[i] = 0x7fffffff; }
        }
    }
}

template <int NV4, int SMAX>
static void expand_reg_launch(hipStream_t st, const Dims &d, int pairs, const float *logits, AView A, RowView rv,
                              float *row_lc, float *dphi, float *cand_score, int *cand_tok, float *row_stats,
                              float *delta_nb) {
    hipLaunchKernelGGL((k_expand_reg<NV4, SMAX>), dim3(pairs), dim3(EXP_THREADS), 0, st, d, logits, A, rv, row_lc, dphi,
                       cand_score, cand_tok, row_stats, delta_nb);
}

hipError_t launch_expand(hipStream_t st, const Dims &d, int pairs, const float *logits, AView A, RowView rv,
                         float *row_lc, float *dphi, float *cand_score, int *cand_tok, float *row_stats,
                         float *delta_nb, int force_generic) {
    if (pairs <= 0) return hipSuccess;
    size_t shm = (size_t)d.V * sizeof(float);
    if (d.V % 4 == 0 && !force_generic) {
#define TBS_EXPAND_REG(NV4, SMAX)                                                                              \
    {                                                                                                          \
        expand_reg_launch<NV4, SMAX>(st, d, pairs, logits, A, rv, row_lc, dphi, cand_score, cand_tok, row_stats, \
                                     delta_nb);                                                                \
        return hipGetLastError();                                                                              \
    }
        const int nv4 = (d.V / 4 + EXP_THREADS - 1) / EXP_THREADS;
        if (nv4 <= 1 && d.S <= 4) TBS_EXPAND_REG(1, 4)
        if (nv4 <= 1 && d.S <= 16) TBS_EXPAND_REG(1, 16)
        if (nv4 <= 2 && d.S <= 8) TBS_EXPAND_REG(2, 8)
        if (nv4 <= 4 && d.S <= 3) TBS_EXPAND_REG(4, 3)
        if (nv4 <= 4 && d.S <= 5) TBS_EXPAND_REG(4, 5)
#undef TBS_EXPAND_REG
    }
    if (d.V % 4 == 0)
        hipLaunchKernelGGL(k_expand<true>, dim3(pairs), dim3(EXP_THREADS), shm, st, d, logits, A, rv, row_lc, dphi,
                           cand_score, cand_tok, row_stats, delta_nb);
    else
        hipLaunchKernelGGL(k_expand<false>, dim3(pairs), dim3(EXP_THREADS), shm, st, d, logits, A, rv, row_lc, dphi,
                           cand_score, cand_tok, row_stats, delta_nb);
    return hipGetLastError();
}
