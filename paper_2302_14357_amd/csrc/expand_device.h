// Device code of the expansion step (Eq. 3-7 and the N best expansions of one hypothesis) shared by
// the kernel that expands every hypothesis of a joiner call and the kernel that runs a whole round
// of one utterance.  The hypothesis is worked on by a team of TT threads (TT/64 waves) that may be a
// whole workgroup or a part of one; barriers are workgroup-wide, so every team of a workgroup must
// call expand_pair together.
#pragma once
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


// Forward variable of Eq. 3 with extended range.  With blank probabilities of a few percent the
// products of Eq. 3 leave the range of float after ~25 frames, while the blank expansion they end
// in (Eq. 7) is still compared with the threshold and kept in B.  alpha is therefore carried as
// m * 2^e, m renormalised to [0.5, 1) at every frame:
//     alpha_t = alpha_{t-1} b_{t-1} + d_old[t]
// For the same reason d_old itself arrives as logarithms: d_old[t] of a token emitted late in a
// long segment is tiny, but it is multiplied by correspondingly few blanks, so every frame
// contributes alike to the blank expansion.
struct ScanAlpha {
    float m;
    int e;
    __device__ __forceinline__ void start() { m = 0.f; e = 0; }
    // logd = log d_old[t] (-inf: no mass at this frame)
    __device__ __forceinline__ void step(float bprev, float logd) {
        m *= bprev;
        if (logd > -INFINITY) {
            // d_old[t] = md * 2^kd with md in [0.5, 1)
            const float l2 = logd * 1.44269504088896341f;
            const float fl = floorf(l2);
            const int kd = (int)fl + 1;
            const float md = __builtin_amdgcn_exp2f(l2 - fl - 1.f);
            if (m == 0.f || e < kd - 40) {   // what came before is below 2^-40 of d_old: beyond float
                m = md;
                e = kd;
            } else {
                m += ldexpf(md, kd - e);     // kd - e <= 40; far below, d_old[t] vanishes instead
            }
        }
        int k;
        m = frexpf(m, &k);
        e += k;
    }
    // log(alpha): natural logarithm, -inf for zero
    __device__ __forceinline__ float log_value() const {
        return m > 0.f ? __logf(m) + (float)e * 0.69314718055994531f : -INFINITY;
    }
    __device__ __forceinline__ float value() const { return ldexpf(m, e); }   // may underflow to 0
    // log(alpha * b): natural logarithm of Eq. 7
    __device__ __forceinline__ float log_times(float b) const {
        const float x = m * b;
        return x > 0.f ? __logf(x) + (float)e * 0.69314718055994531f : -INFINITY;
    }
};

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

// ------------------------------------------------------------------ register-resident variant
// When the S' x V logits of one hypothesis fit in the registers of one workgroup
// (V <= 1024 NV4 columns, S' <= SMAX), every logit is read from memory exactly
// once and exponentiated exactly once: the row maxima m_t are reduced across the
// workgroup first, each thread then keeps e = exp(l - m_t) of its own columns,
// the row sums Z_t follow from one more reduction, and the streaming sum of
// Eq. 4-6 becomes delta_nb[k] = sum_t c_t e[t][k] from registers.  The N best
// are then taken per wave from registers and merged by the first wave.
//
// The arithmetic per logit is one exp, one multiply-add for the exponent and two
// for the sums; everything else below is bookkeeping per wave, and at four waves
// per hypothesis that bookkeeping costs as many issue cycles as the logits do.  It
// is therefore written to be short: reductions in the integer domain or with the
// DPP operand folded into the add, thresholds and ranks by counting against lane
// values broadcast through scalar registers instead of rounds of arg-max.
template <int SMAX, int TW>
struct ExpandShared {
    float pm[SMAX][TW], pz[SMAX][TW];   // per-wave row maxima and row sums
    float cv[TW][EXP_CAND_CAP];   // candidates of each wave ...
    int ck[TW][EXP_CAND_CAP];
    float jv[TW * EXP_CAND_CAP];  // ... and all of them in one list, in any order
    int jk[TW * EXP_CAND_CAP];
    int jn;                              // entries of the joint list
};

// What a workgroup needs to know of one (utterance, hypothesis) pair besides its logits.
template <int SMAX>
struct ExpandPair {
    int pair, row0, sp;
    float dold[SMAX];   // frame distribution of the hypothesis' last token (d_old of Eq. 3), as logarithms
    float lblank[SMAX]; // blank logit of each row
};

// Row lists, d_old and the logits are written by earlier kernels only: what every lane needs alike
// is read through the constant address space, so that a wave-uniform address becomes a scalar
// load into scalar registers.
typedef const __attribute__((address_space(4))) int *cint_p;
typedef const __attribute__((address_space(4))) float *cfloat_p;

// (the caller knows the pair's rows and place: nothing is read from the pair list)
template <int SMAX>
__device__ __forceinline__ void expand_pair_info_at(ExpandPair<SMAX> &pi, int pair, int row0, int sp, int u, int h,
                                                    const Dims &d, const AView &A, const float *logits) {
    pi.pair = pair;
    pi.row0 = row0;
    pi.sp = sp;
    cfloat_p dold = (cfloat_p)A.dhat + ((long)u * d.N + h) * d.S;
#pragma unroll
    for (int t = 0; t < SMAX; ++t) pi.dold[t] = t < pi.sp ? dold[t] : -INFINITY;
    cfloat_p lb = (cfloat_p)logits + (long)pi.row0 * d.V + d.blank;
#pragma unroll
    for (int t = 0; t < SMAX; ++t) pi.lblank[t] = t < pi.sp ? lb[(long)t * d.V] : 0.f;
}

template <int SMAX>
__device__ __forceinline__ void expand_pair_info(ExpandPair<SMAX> &pi, int pair, const Dims &d, const AView &A,
                                                 const RowView &rv, const float *logits) {
    pi.pair = pair;
    pi.row0 = ((cint_p)rv.pair_row0)[pair];
    pi.sp = ((cint_p)rv.pair_len)[pair];
    const int u = ((cint_p)rv.pair_u)[pair], h = ((cint_p)rv.pair_h)[pair];
    cfloat_p dold = (cfloat_p)A.dhat + ((long)u * d.N + h) * d.S;
#pragma unroll
    for (int t = 0; t < SMAX; ++t) pi.dold[t] = t < pi.sp ? dold[t] : -INFINITY;
    cfloat_p lb = (cfloat_p)logits + (long)pi.row0 * d.V + d.blank;
#pragma unroll
    for (int t = 0; t < SMAX; ++t) pi.lblank[t] = t < pi.sp ? lb[(long)t * d.V] : 0.f;
}

// One pass over memory: this thread's columns of every row of the pair.  Every request is made
// whatever S' and V are (rows past S' repeat the last row, columns past V the last column group;
// expand_pair discards them), so that the loads are straight-line code with scalar row bases.
template <int NV4, int SMAX, int TT>
__device__ __forceinline__ void expand_load(float (&e)[SMAX][NV4 * 4], const float *__restrict__ logits, int row0,
                                            int sp, int V, int tid) {
    const int V4 = V >> 2;
    unsigned off[NV4];   // byte offsets within a row
#pragma unroll
    for (int q = 0; q < NV4; ++q) off[q] = 16u * (unsigned)min(tid + TT * q, V4 - 1);
#pragma unroll
    for (int t = 0; t < SMAX; ++t) {
        const char *row = reinterpret_cast<const char *>(logits + ((long)row0 + max(min(t, sp - 1), 0)) * V);
#pragma unroll
        for (int q = 0; q < NV4; ++q) {
            const float4 x = *reinterpret_cast<const float4 *>(row + off[q]);
            e[t][4 * q + 0] = x.x; e[t][4 * q + 1] = x.y; e[t][4 * q + 2] = x.z; e[t][4 * q + 3] = x.w;
        }
    }
}

// floats as integers of the same order (and back: the map is its own inverse)
__device__ __forceinline__ int f2ord(float f) {
    const int b = __float_as_int(f);
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float ord2f(int i) { return __int_as_float(i ^ ((i >> 31) & 0x7fffffff)); }

// wave maximum through the integer order: the DPP operand folds into v_max_i32 and the four
// row results combine on the scalar unit
__device__ __forceinline__ float wave_max_ord(float f) {
    int v = f2ord(f);
    v = max(v, dpp_i<DPP_QUAD_SWAP1>(v));
    v = max(v, dpp_i<DPP_QUAD_SWAP2>(v));
    v = max(v, dpp_i<DPP_HALF_MIRROR>(v));
    v = max(v, dpp_i<DPP_MIRROR>(v));
    return ord2f(max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
                     max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48))));
}

// (expand_pair meets the other teams of its workgroup at this many barriers; a wave of the workgroup
// that does something else meanwhile must meet them too)
#define EXPAND_PAIR_BARRIERS 3

// Everything after the load for one pair, by a team of TT threads (tid = 0 .. TT-1 within the team).
// Results: lc_out[t] = log(alpha_t / Z_t) - m_t for the pair's frames, *dphi_out = log of the blank
// expansion relative to the hypothesis score, cs / ct = logarithms and tokens of the N best
// expansions in order (-inf / -1 where there are fewer); any of them may point into LDS.
// live = false: a team with no hypothesis; it only keeps the workgroup's barriers company.
template <int NV4, int SMAX, int TT>
__device__ __forceinline__ void expand_pair(float (&e)[SMAX][NV4 * 4], const ExpandPair<SMAX> &pi,
                                            ExpandShared<SMAX, TT / 64> &sm, const Dims &d, int tid, bool live,
                                            float *lc_out, float *dphi_out, float *cs, int *ct,
                                            float *__restrict__ row_stats, float *__restrict__ delta_nb) {
    constexpr int NC = NV4 * 4;  // columns per thread
    constexpr int TW = TT / 64;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int V = d.V, V4 = V >> 2;
    // Rows past S' and columns past V hold copies of real logits (see expand_load): copies leave a
    // row maximum unchanged, the row sums skip the copied columns, the copied rows get coefficient
    // zero and the copied columns score zero below.
    float mrow[SMAX];
#pragma unroll
    for (int t = 0; t < SMAX; ++t) {
        mrow[t] = -INFINITY;
#pragma unroll
        for (int c = 0; c < NC; ++c) mrow[t] = fmaxf(mrow[t], e[t][c]);
    }
    // ---- row maxima across the workgroup (waves by DPP, then through LDS)
#pragma unroll
    for (int t = 0; t < SMAX; ++t) {
        const float m = wave_max_ord(mrow[t]);
        if (lane == 0) sm.pm[t][wave] = m;
    }
    if (tid == 0) sm.jn = 0;
    __syncthreads();
#pragma unroll
    for (int t = 0; t < SMAX; ++t) {
        float m = sm.pm[t][0];
#pragma unroll
        for (int w = 1; w < TW; ++w) m = fmaxf(m, sm.pm[t][w]);
        if (SMAX * TW > 8) __builtin_amdgcn_sched_barrier(0);   // one row at a time: the partial results of many rows at once cost registers
        mrow[t] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(m)));   // uniform: a scalar register
    }
    // ---- e = exp(l - m_t), once per logit; row sums across the workgroup
#pragma unroll
    for (int t = 0; t < SMAX; ++t) {
        const float nm = -mrow[t] * 1.44269504088896341f;
        float z = 0.f;
#pragma unroll
        for (int q = 0; q < NV4; ++q) {
            float zq = 0.f;
#pragma unroll
            for (int c = 4 * q; c < 4 * q + 4; ++c) {
                e[t][c] = __builtin_amdgcn_exp2f(fmaf(e[t][c], 1.44269504088896341f, nm));
                zq += e[t][c];
            }
            z += (tid + TT * q < V4) ? zq : 0.f;
        }
        z = wave_sum(z);
        if (lane == 0) sm.pz[t][wave] = z;
    }
    __syncthreads();
    // ---- every thread: row sums, forward variable (Eq. 3 as a scan), Eq. 7, the row coefficients.
    // The scan runs on logarithms: la_t = log alpha_t = logaddexp(la_{t-1} + log b_{t-1}, log d_old[t]),
    // which has the range the products of Eq. 3 need (see ScanAlpha) at four transcendentals and a
    // dozen plain operations per frame; the values are the same in every lane.  What goes to memory
    // is kept in registers until the scan is over and then stored by one thread in one go.
    float cf[SMAX], lcrow[SMAX];
    float lphi = -INFINITY;
    {
        float la = -INFINITY, lbprev = 0.f;
#pragma unroll
        for (int t = 0; t < SMAX; ++t) {
            cf[t] = 0.f;
            lcrow[t] = 0.f;
            if (t < pi.sp) {   // (uniform)
                float z = sm.pz[t][0];
#pragma unroll
                for (int w = 1; w < TW; ++w) z += sm.pz[t][w];
                __builtin_amdgcn_sched_barrier(0);
                const float lz = __logf(z);
                const float lb = (pi.lblank[t] - mrow[t]) - lz;       // log of the blank probability of frame t
                const float x = la + lbprev, ld = pi.dold[t];
                const float mx = fmaxf(x, ld), mn = fminf(x, ld);
                la = mx > -INFINITY ? mx + __logf(1.f + __expf(mn - mx)) : -INFINITY;
                lbprev = lb;
                const float lc = la - lz;                              // log(alpha_t / Z_t)
                cf[t] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(__expf(lc))));
                lcrow[t] = lc - mrow[t];
                if (t == pi.sp - 1) lphi = la + lb;                    // Eq. 7
                if (row_stats && tid == 0 && live) {
                    row_stats[(long)(pi.row0 + t) * 3 + 0] = mrow[t];
                    row_stats[(long)(pi.row0 + t) * 3 + 1] = z;
                    row_stats[(long)(pi.row0 + t) * 3 + 2] = __expf(lb);
                }
            }
        }
    }
    if (tid == 0 && live) {
#pragma unroll
        for (int t = 0; t < SMAX; ++t)
            if (t < pi.sp) lc_out[t] = lcrow[t];   // log(alpha_t / Z_t) - m_t
        *dphi_out = lphi;
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
    // blank is not a non-blank expansion; columns past V do not exist.  (Blank in column 0 and a
    // vocabulary that fills every thread's columns, the usual case, cost one select; anything
    // else takes the general form.)
    if (d.blank == 0 && V4 == TT * NV4) {   // (uniform)
        if (tid == 0) v[0] = 0.f;
    } else {
#pragma unroll
        for (int q = 0; q < NV4; ++q)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int col = 4 * (tid + TT * q) + c;
                if (col == d.blank || col >= V) v[4 * q + c] = 0.f;
            }
    }
    if (delta_nb && live) {   // debug output: its indices are made afresh, not kept in registers from the loads
        int t2 = tid;
        asm volatile("" : "+v"(t2));
#pragma unroll
        for (int q = 0; q < NV4; ++q) {
            const int i4 = t2 + TT * q;
            if (i4 < V4)
                reinterpret_cast<float4 *>(delta_nb + (long)pi.pair * V)[i4] =
                    make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
        }
    }
    // ---- candidates of this wave: every score >= tau, where tau is a lower bound of the wave's
    // N-th largest score (ties included, so usually only a few more than N qualify).  Scores are
    // positive floats, ordered like their bit patterns.
    float tau;
    {
        float lm = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) lm = fmaxf(lm, v[c]);
        if (d.N <= 16) {
            // N-th largest of the 16 quad maxima: each is a score of this wave, so the N-th largest
            // of them cannot exceed the N-th largest of all.  The low four bits of a key give way to
            // the quad's number, which makes the keys distinct; every lane counts the keys above its
            // own, and the quad that counts N-1 holds the threshold (rounded down by those bits).
            unsigned key = __float_as_uint(lm);
            key = max(key, (unsigned)dpp_i<DPP_QUAD_SWAP1>((int)key));
            key = max(key, (unsigned)dpp_i<DPP_QUAD_SWAP2>((int)key));
            key = (key & ~15u) | (unsigned)(15 - (lane >> 2));
            int above = 0;
#pragma unroll
            for (int g = 0; g < 16; ++g) above += (unsigned)__builtin_amdgcn_readlane((int)key, 4 * g) > key;
            const u64 at = __ballot(above == d.N - 1);
            const unsigned kth = (unsigned)__builtin_amdgcn_readlane((int)key, __ffsll((long long)at) - 1);
            tau = __uint_as_float(kth & ~15u);
        } else {
            // N rounds of wave maximum over the thread maxima, one lane retiring per round
            tau = 0.f;
            for (int n = 0; n < d.N; ++n) {
                tau = wave_max(lm);
                if (!(tau > 0.f)) break;   // fewer than N positive maxima: every positive score qualifies
                const u64 holders = __ballot(lm == tau);
                if (lane == __ffsll((long long)holders) - 1) lm = -1.f;
            }
        }
        // the smallest normal float stands for "any positive score"
        tau = fmaxf(tau, 1.17549435e-38f);
    }
    int total = 0;
    {
#pragma unroll
        for (int q = 0; q < NV4; ++q)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float x = v[4 * q + c];
                const bool take = x >= tau;
                const u64 m = __ballot(take);
                if (m) {   // uniform
                    const int pos = total + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32),
                                                                           __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
                    if (take && pos < EXP_CAND_CAP) {
                        sm.cv[wave][pos] = x;
                        sm.ck[wave][pos] = 4 * (tid + TT * q) + c;
                    }
                    total += __popcll(m);
                }
            }
    }
    if (total > EXP_CAND_CAP) {
        // many equal scores: take exactly the N best by N rounds of wave arg-max
        total = 0;
        for (int n = 0; n < d.N; ++n) {
            float bv = 0.f;
            int bk = 0x7fffffff;
#pragma unroll
            for (int q = 0; q < NV4; ++q)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float x = v[4 * q + c];
                    if (x > bv) { bv = x; bk = 4 * (tid + TT * q) + c; }   // ascending columns
                }
            wave_argmax(bv, bk);
            if (!(bv > 0.f)) break;
            if (lane == 0) { sm.cv[wave][n] = bv; sm.ck[wave][n] = bk; }
            total = n + 1;
#pragma unroll
            for (int q = 0; q < NV4; ++q)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (4 * (tid + TT * q) + c == bk) v[4 * q + c] = -1.f;
        }
    }
    // append this wave's list to the joint list (the order of waves there does not matter: the
    // merge below orders by score and token)
    {
        int base = 0;
        if (lane == 0) base = atomicAdd(&sm.jn, total);
        base = __builtin_amdgcn_readfirstlane(base);
        if (lane < total) {
            sm.jv[base + lane] = sm.cv[wave][lane];
            sm.jk[base + lane] = sm.ck[wave][lane];
        }
    }
    __syncthreads();
    // ---- merge (first wave): larger score first, smaller token on equal scores
    if (wave == 0 && live) {
        const int all = sm.jn;
        if (all <= 64) {
            // one candidate per lane, as a 64-bit key (score bits, inverted token) that orders like
            // the rule above; the rank of a candidate is the number of keys above its own
            const bool have = lane < all;
            const float x = have ? sm.jv[lane] : 0.f;
            const int k = have ? sm.jk[lane] : 0x7fffffff;
            const u64 key = ((u64)__float_as_uint(x) << 32) | (unsigned)(0x7fffffff - k);
            int rank = 0;
            for (int j = 0; j < all; ++j) {
                const u64 kj = ((u64)(unsigned)__builtin_amdgcn_readlane((int)(key >> 32), j) << 32) |
                               (unsigned)__builtin_amdgcn_readlane((int)key, j);
                rank += kj > key;
            }
            if (have && rank < d.N) { cs[rank] = __logf(x); ct[rank] = k; }
            if (lane >= all && lane < d.N) { cs[lane] = -INFINITY; ct[lane] = -1; }
        } else {
            float cv[TW];
            int ck[TW];
#pragma unroll
            for (int i = 0; i < TW; ++i) {
                const bool have = lane + 64 * i < all;
                cv[i] = have ? sm.jv[lane + 64 * i] : -1.f;
                ck[i] = have ? sm.jk[lane + 64 * i] : 0x7fffffff;
            }
            for (int n = 0; n < d.N; ++n) {
                float bv = -1.f;
                int bk = 0x7fffffff;
#pragma unroll
                for (int i = 0; i < TW; ++i)
                    if (cv[i] > bv || (cv[i] == bv && ck[i] < bk)) { bv = cv[i]; bk = ck[i]; }
                wave_argmax(bv, bk);
                if (lane == 0) {
                    const bool ok = bv > 0.f && bk != 0x7fffffff;
                    cs[n] = ok ? __logf(bv) : -INFINITY;
                    ct[n] = ok ? bk : -1;
                }
#pragma unroll
                for (int i = 0; i < TW; ++i)
                    if (ck[i] == bk) { cv[i] = -1.f; ck[i] = 0x7fffffff; }
            }
        }
    }
}

