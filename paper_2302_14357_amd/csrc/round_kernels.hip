// One round of the inner loop of Algorithm 1 behind the joiner, for small shapes, as one kernel:
// a workgroup per utterance expands all of the utterance's live hypotheses at once (Eq. 3-7 and the
// N best expansions of each, one team of 64 to 256 threads per hypothesis), hands the results to
// its first wave through LDS, and that wave does AddAndMerge, ChooseNthScore, the joint
// ChooseNBestExpansions with the threshold test and the new list A.  Where the logits of one
// utterance's hypotheses (at most N * S' * V values) fit the registers of one workgroup this saves a
// kernel boundary and the trip of the candidates through memory in every round of a decode whose
// time is the length of its chain of dependent kernels.
#include "expand_device.h"
#include "select_device.h"

template <int TW, int NV4, int SMAX>
__global__ void __launch_bounds__(1024)
k_round(Dims d, int round, int drop, const float *__restrict__ logits, AView A, AView An, BView B, RowView rv,
        const int2 *nodes, float *__restrict__ row_stats, float *__restrict__ delta_nb) {
    constexpr int TT = TW * 64;
    typedef ExpandShared<SMAX, TW> TeamShared;
    extern __shared__ __attribute__((aligned(16))) unsigned char s_raw[];
    // LDS: the utterance's B list for the select step, one TeamShared per team, then what the teams
    // hand to the select step
    const int N = d.N;
    const size_t b_list = ((size_t)d.BCAP * (sizeof(double) + sizeof(u64) + 3 * sizeof(int)) + 15) & ~(size_t)15;
    TeamShared *teams = reinterpret_cast<TeamShared *>(s_raw + b_list);
    float *s_lc = reinterpret_cast<float *>(teams + N);   // [H, S']
    float *s_dphi = s_lc + N * SMAX;                       // [H]
    float *s_cs = s_dphi + N;                              // [H, N]
    int *s_ct = reinterpret_cast<int *>(s_cs + N * N);     // [H, N]

    const int u = blockIdx.x;
    const int team = __builtin_amdgcn_readfirstlane((int)threadIdx.x / TT), tid = (int)threadIdx.x % TT;
    const int sp = rv.utt_sp[u];
    const int H = sp > 0 ? A.count[u] : 0;
    if (H == 0) {   // (the same for the whole workgroup: nobody reaches a barrier)
        if (threadIdx.x == 0) An.count[u] = 0;
        return;
    }
    const int pair0 = rv.utt_pair0[u];
    const bool live = team < H;
    ExpandPair<SMAX> pi;
    if (live) {
        expand_pair_info(pi, pair0 + team, d, A, rv, logits);
    } else {   // a team without a hypothesis reads the utterance's first row and scores nothing
        pi.pair = pair0;
        pi.row0 = rv.utt_row0[u];
        pi.sp = 0;
#pragma unroll
        for (int t = 0; t < SMAX; ++t) {
            pi.dold[t] = -INFINITY;
            pi.lblank[t] = 0.f;
        }
    }
    float e[SMAX][NV4 * 4];
    expand_load<NV4, SMAX, TT>(e, logits, pi.row0, pi.sp, d.V, tid);
    expand_pair<NV4, SMAX, TT>(e, pi, teams[team], d, tid, live, s_lc + team * sp, s_dphi + team, s_cs + team * N,
                               s_ct + team * N, row_stats, delta_nb);
    __syncthreads();
    if (threadIdx.x < WAVE) {
        SelectIn in;
        in.cand_score = s_cs;
        in.cand_tok = s_ct;
        in.dphi = s_dphi;
        in.lc = s_lc;
        select_merge_utt(d, round, drop, u, (int)threadIdx.x, logits, in, A, An, B, rv, nodes, s_raw);
    }
}

// which instantiation serves the shape (0 = none): hypotheses per workgroup x threads per hypothesis
// stay within 1024 threads, a hypothesis' S x V logits within its team's registers
static int round_variant(const Dims &d) {
    if (d.V % 4 || d.S > 5 || d.N > 16) return 0;
    const int tw = d.N <= 4 ? 4 : (d.N <= 8 ? 2 : 1);
    const int nv4 = tw == 4 ? 1 : (tw == 2 ? 2 : 4);
    if (d.V / 4 > tw * 64 * nv4) return 0;
    return tw * 10 + (d.S <= 3 ? 3 : 5);
}

bool round_fits(const Dims &d) { return round_variant(d) != 0; }

template <int TW, int NV4, int SMAX>
static hipError_t round_launch(hipStream_t st, const Dims &d, int round, int drop, const float *logits, AView A,
                               AView An, BView B, RowView rv, const int2 *nodes, float *row_stats, float *delta_nb) {
    const size_t b_list = ((size_t)d.BCAP * (sizeof(double) + sizeof(u64) + 3 * sizeof(int)) + 15) & ~(size_t)15;
    const size_t shm = b_list + (size_t)d.N * sizeof(ExpandShared<SMAX, TW>) +
                       sizeof(float) * ((size_t)d.N * SMAX + d.N + 2 * (size_t)d.N * d.N);
    static size_t attr_for = 0;
    if (shm > attr_for) {   // (static LDS of the select step comes on top: raise the limit to what the launch needs)
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_round<TW, NV4, SMAX>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) return e;
        attr_for = shm;
    }
    hipLaunchKernelGGL((k_round<TW, NV4, SMAX>), dim3(d.U), dim3(d.N * TW * 64), shm, st, d, round, drop, logits, A, An,
                       B, rv, nodes, row_stats, delta_nb);
    return hipGetLastError();
}

hipError_t launch_round(hipStream_t st, const Dims &d, int round, int drop, const float *logits, AView A, AView An,
                        BView B, RowView rv, const int2 *nodes, float *row_stats, float *delta_nb) {
    switch (round_variant(d)) {
        case 43: return round_launch<4, 1, 3>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb);
        case 45: return round_launch<4, 1, 5>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb);
        case 23: return round_launch<2, 2, 3>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb);
        case 25: return round_launch<2, 2, 5>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb);
        case 13: return round_launch<1, 4, 3>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb);
        case 15: return round_launch<1, 4, 5>(st, d, round, drop, logits, A, An, B, rv, nodes, row_stats, delta_nb);
        default: return hipErrorInvalidValue;
    }
}
