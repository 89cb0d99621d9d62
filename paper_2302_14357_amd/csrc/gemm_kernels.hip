// bf16 MFMA GEMM of the joiner (and of the predictor's dense layers):
//   C[M,N] = A[M,K] * B[N,K]^T + bias[N],  bf16 inputs, fp32 accumulate, fp32 output
// (optionally rows scattered through out_row, and a per-row bias gathered from a table).
//
// Workgroup = WM x WN waves; each wave owns TM x TN blocks of 32x32 computed
// with v_mfma_f32_32x32x16_bf16, so a workgroup tile is (32 TM WM) x (32 TN WN).
// K is consumed in tiles of 64 through LDS.  LDS rows are 128 bytes (8 chunks
// of 16 bytes) and chunk c of row r is stored at position c ^ (r & 7): the
// 16-byte fragment reads of 8 consecutive rows then touch 8 different chunk
// positions, i.e. all banks once, with no padding.  Two LDS buffers alternate,
// the next K tile is fetched from global memory into registers while the
// current one is multiplied, and one barrier per K tile separates them.
// The grid is one-dimensional and maps workgroups to tiles so that the
// workgroups resident on one XCD (ids equal modulo 8) work on a compact block of
// tiles and share their operand rows in that XCD's L2.
#include "tbs_internal.h"
#include <climits>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

#define GEMM_XCDS 8
#define GEMM_GROUP_M 8   // M tiles per XCD block (measured: 4 -> 8 is +6..10 % at 25600..51200 rows, B is re-read per block)

// LDS rows hold BK bf16 = BK/8 chunks of 16 bytes; chunk c of row r sits at position c ^ swz(r).
// A 16-byte-per-lane LDS read is served 16 lanes (256 bytes = all 64 banks) per cycle, so 16
// consecutive rows reading the same chunk must land on 16 different (position, row parity)
// places: 128-byte rows need 8 positions changing every second row, 256-byte rows 16 positions.
template <int BK>
__device__ __forceinline__ int gemm_swz(int row) {
    return BK == 64 ? ((row >> 1) & 7) : (row & 15);
}

// Position idx of XCD xcd's tile sequence -> (tile_m, tile_n).  Tiles are ordered
// in blocks of GEMM_GROUP_M rows of tiles (M fastest inside a block) and XCD x
// owns the x-th contiguous eighth of that order, so the workgroups resident on
// one XCD at any time work on neighbouring tiles.
__device__ __forceinline__ bool gemm_tile_of(int xcd, int idx, int tiles_m, int tiles_n, int group_m, int &tm, int &tn) {
    const int total = tiles_m * tiles_n;
    const int chunk = (total + GEMM_XCDS - 1) / GEMM_XCDS;
    const int t = xcd * chunk + idx;
    tm = 0;
    tn = 0;
    if (idx >= chunk || t >= total) return false;
    const int per_block = group_m * tiles_n;
    const int b = t / per_block, r = t % per_block;
    const int gm = min(group_m, tiles_m - b * group_m);
    tm = b * group_m + r % gm;
    tn = r / gm;
    return true;
}

// Persistent kernel: gridDim.x (a multiple of 8) workgroups each walk a strided
// share of their XCD's tile sequence.  The first K tile of the next output tile
// is prefetched during the last K tile of the current one and the epilogue's
// stores are left in flight, so neither the load latency at the head of a tile
// nor the store traffic at its tail stalls the matrix cores.
template <int TM, int TN, int WM, int WN, int BK, bool KGUARD>
__global__ void __launch_bounds__(64 * WM * WN)
k_gemm_bf16(const bf16_t *__restrict__ A, const bf16_t *__restrict__ B, const float *__restrict__ bias,
            float *__restrict__ C, int M, int N, int K, const int *__restrict__ out_row, long ldc, int tiles_m,
            int tiles_n, int group_m, const int *__restrict__ m_begin, const int *__restrict__ m_end) {
    constexpr int NT = 64 * WM * WN;
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    constexpr int CH = BK / 8;                                       // 16-byte chunks per LDS row
    constexpr int A_CHUNKS = BM * CH / NT, B_CHUNKS = BN * CH / NT;  // chunks per thread per K tile
    constexpr int ROWS_PER_PASS = NT / CH;
    constexpr int TILE_ELEMS = (BM + BN) * BK;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];   // 2 x [A tile | B tile]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int xcd = blockIdx.x % GEMM_XCDS, jstride = gridDim.x / GEMM_XCDS;
    int idx = blockIdx.x / GEMM_XCDS;
    if (m_begin) {
        // a piece of a larger product: its rows [*m_begin, *m_end) are known on the device only (the
        // launch was sized for the most the piece can hold); operands and result shift to the piece
        const int mb = *m_begin, me = *m_end;
        A += (long)mb * K;
        C += (long)mb * ldc;
        M = me - mb;
        if (M <= 0) return;
        tiles_m = (M + BM - 1) / BM;
    }
    int tile_m, tile_n;
    if (!gemm_tile_of(xcd, idx, tiles_m, tiles_n, group_m, tile_m, tile_n)) return;

    floatx16 acc[TM][TN];

    // chunk (row, kc) this thread moves per pass, and where it lands in an LDS buffer
    const int kc = tid % CH, crow = tid / CH;
    int la[A_CHUNKS], lb[B_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
        int row = crow + ROWS_PER_PASS * i;
        la[i] = row * BK + ((kc ^ gemm_swz<BK>(row)) * 8);
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
        int row = crow + ROWS_PER_PASS * i;
        lb[i] = BM * BK + row * BK + ((kc ^ gemm_swz<BK>(row)) * 8);
    }
    // global sources of the current tile (rows clamped, so reads stay in bounds)
    // Without a K guard the tiles go from global memory straight into LDS (no registers in
    // between): lane l of a wave always fills LDS slot l of the wave's 1 KB destination, so it is
    // the global chunk that is chosen per lane: slot position p of row r receives chunk p ^ swz(r).
    constexpr bool DIRECT = !KGUARD;
    const int kcg = DIRECT ? (kc ^ gemm_swz<BK>(crow)) : kc;   // ROWS_PER_PASS is a multiple of 16
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const bf16_t *ga[A_CHUNKS], *gb[B_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i)
        ga[i] = A + (long)min(tile_m * BM + crow + ROWS_PER_PASS * i, M - 1) * K + kcg * 8;
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i)
        gb[i] = B + (long)min(tile_n * BN + crow + ROWS_PER_PASS * i, N - 1) * K + kcg * 8;

    // fragment addresses: lane reads row (lane & 31) of a 32-row block, K chunk 2*kk + (lane >> 5)
    const int frow = lane & 31, fsel = lane >> 5;
    int fa[TM], fb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = (wm * 32 * TM + i * 32 + frow) * BK;
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[j] = BM * BK + (wn * 32 * TN + j * 32 + frow) * BK;
    const int fsw = gemm_swz<BK>(frow);

    const int ktiles = (K + BK - 1) / BK;
    uint4 ra[A_CHUNKS], rb[B_CHUNKS];
    // prologue: K tile 0 of the first tile -> LDS buffer 0
    if (DIRECT) {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)ga[i],
                                             (__attribute__((address_space(3))) void *)(smem + (i * NT + wave_u * 64) * 8),
                                             16, 0, 0);
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gb[i],
                                             (__attribute__((address_space(3))) void *)(smem + BM * BK + (i * NT + wave_u * 64) * 8),
                                             16, 0, 0);
        __builtin_amdgcn_s_waitcnt(0);
    } else {
        const bool in = kc * 8 < K;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) ra[i] = in ? *reinterpret_cast<const uint4 *>(ga[i]) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) rb[i] = in ? *reinterpret_cast<const uint4 *>(gb[i]) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<uint4 *>(smem + la[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) *reinterpret_cast<uint4 *>(smem + lb[i]) = rb[i];
    }
    __syncthreads();
    int buf = 0;
    for (;;) {
        // accumulators start from the bias: a lane's column is the same for all 16 of its entries
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = tile_n * BN + wn * 32 * TN + j * 32 + (lane & 31);
            const float bv = (bias && col < N) ? bias[col] : 0.f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = bv;
        }
        // the tile after this one (if any): its first K tile is prefetched at the end of this one
        int next_m, next_n;
        const bool have_next = gemm_tile_of(xcd, idx + jstride, tiles_m, tiles_n, group_m, next_m, next_n);
        const bf16_t *gan[A_CHUNKS], *gbn[B_CHUNKS];
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i)
            gan[i] = have_next ? A + (long)min(next_m * BM + crow + ROWS_PER_PASS * i, M - 1) * K + kcg * 8 : ga[i];
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i)
            gbn[i] = have_next ? B + (long)min(next_n * BN + crow + ROWS_PER_PASS * i, N - 1) * K + kcg * 8 : gb[i];

        for (int kt = 0; kt < ktiles; ++kt) {
            const bf16_t *cur = smem + buf * TILE_ELEMS;
            bf16_t *nxt = smem + (buf ^ 1) * TILE_ELEMS;
            const bool last = kt + 1 == ktiles;
            const int kn = last ? 0 : (kt + 1) * BK;
            if (DIRECT) {
#pragma unroll
                for (int i = 0; i < A_CHUNKS; ++i)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)((last ? gan[i] : ga[i]) + kn),
                        (__attribute__((address_space(3))) void *)(nxt + (i * NT + wave_u * 64) * 8), 16, 0, 0);
#pragma unroll
                for (int i = 0; i < B_CHUNKS; ++i)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)((last ? gbn[i] : gb[i]) + kn),
                        (__attribute__((address_space(3))) void *)(nxt + BM * BK + (i * NT + wave_u * 64) * 8), 16, 0, 0);
            } else {
                const bool in = kn + kc * 8 < K;
#pragma unroll
                for (int i = 0; i < A_CHUNKS; ++i) {
                    const bf16_t *src = (last ? gan[i] : ga[i]) + kn;
                    ra[i] = in ? *reinterpret_cast<const uint4 *>(src) : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < B_CHUNKS; ++i) {
                    const bf16_t *src = (last ? gbn[i] : gb[i]) + kn;
                    rb[i] = in ? *reinterpret_cast<const uint4 *>(src) : make_uint4(0, 0, 0, 0);
                }
            }
            // keep the prefetch ahead of the multiply: without this fence the compiler sinks the
            // loads down to their first use (the LDS stores below) and exposes their latency
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                bf16x8 af[TM], bfr[TN];
                const int cpos = ((kk * 2 + fsel) ^ fsw) * 8;
#pragma unroll
                for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const bf16x8 *>(cur + fa[i] + cpos);
#pragma unroll
                for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const bf16x8 *>(cur + fb[j] + cpos);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
            }
            // the other buffer was last read one iteration ago, which every wave has left
            if (DIRECT) {
                __builtin_amdgcn_s_waitcnt(0);   // this wave's direct loads have landed in LDS
            } else {
#pragma unroll
                for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<uint4 *>(nxt + la[i]) = ra[i];
#pragma unroll
                for (int i = 0; i < B_CHUNKS; ++i) *reinterpret_cast<uint4 *>(nxt + lb[i]) = rb[i];
            }
            __syncthreads();
            buf ^= 1;
        }

        // epilogue: lane holds column (lane & 31); accumulator r is row 8*(r/4) + 4*(lane/32) + r%4
        const int m0 = tile_m * BM, n0 = tile_n * BN;
        if (out_row == nullptr && m0 + BM <= M && n0 + BN <= N) {
            // interior tile: address = uniform row base (scalar registers) + one per-lane offset
            // + a constant, so a store costs no vector address arithmetic
            const unsigned offl = (unsigned)(wm * 32 * TM + (lane >> 5) * 4) * (unsigned)ldc +
                                  (unsigned)(wn * 32 * TN + (lane & 31));
            float *tb = C + (long)m0 * ldc + n0;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float *tr = tb + (long)(i * 32 + (r >> 2) * 8 + (r & 3)) * ldc;   // uniform
#pragma unroll
                    for (int j = 0; j < TN; ++j) tr[offl + j * 32] = acc[i][j][r];
                }
        } else {
            // edge tiles and scattered rows.  The destination rows of a 32-row block are requested
            // together and waited for once, outside any branch: a load behind a branch makes every
            // later store wait for the store before it.
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                long orow[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = min(m0 + wm * 32 * TM + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3), M - 1);
                    orow[r] = out_row ? out_row[row] : row;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) asm volatile("" : "+v"(orow[r]));
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = n0 + wn * 32 * TN + j * 32 + (lane & 31);
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = m0 + wm * 32 * TM + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                        if (row < M && col < N) {
                            C[orow[r] * ldc + col] = acc[i][j][r];
                        }
                    }
                }
            }
        }
        if (!have_next) break;
        idx += jstride;
        tile_m = next_m;
        tile_n = next_n;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) ga[i] = gan[i];
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) gb[i] = gbn[i];
    }
}

template <int TM, int TN, int WM, int WN, int BK, int OCC>
static hipError_t gemm_launch(hipStream_t st, const bf16_t *A, const bf16_t *B, const float *bias, float *C, int M,
                              int N, int K, const int *out_row, long ldc, const int *m_begin = nullptr,
                              const int *m_end = nullptr) {
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const size_t shm = 2u * (BM + BN) * BK * sizeof(bf16_t);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_bf16<TM, TN, WM, WN, BK, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_bf16<TM, TN, WM, WN, BK, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // one wave of resident workgroups (256 CUs x OCC), a multiple of the 8 XCDs, no more than the tiles
    const long total = (long)tiles_m * tiles_n;
    long g = ((total + GEMM_XCDS - 1) / GEMM_XCDS) * GEMM_XCDS;
    if (g > 256L * OCC) g = 256L * OCC;
    const dim3 grid((unsigned)g), block(64 * WM * WN);
    if (K % BK == 0)
        hipLaunchKernelGGL((k_gemm_bf16<TM, TN, WM, WN, BK, false>), grid, block, shm, st, A, B, bias, C, M, N, K, out_row,
                           ldc, tiles_m, tiles_n, GEMM_GROUP_M, m_begin, m_end);
    else
        hipLaunchKernelGGL((k_gemm_bf16<TM, TN, WM, WN, BK, true>), grid, block, shm, st, A, B, bias, C, M, N, K, out_row,
                           ldc, tiles_m, tiles_n, GEMM_GROUP_M, m_begin, m_end);
    return hipGetLastError();
}

// ------------------------------------------------------------------ small problems
// When the whole product is one wave of 64x64 tiles or less, time is latency, not throughput: a
// workgroup alone on its CU that fetches one K tile ahead waits a full memory round trip per K
// tile.  This kernel asks for up to `ns` K tiles of 128 at once, straight into as many LDS
// stages (32 KB each), and multiplies them as they land; a stage is refilled as soon as every
// wave has read it.  One tile per workgroup, 4 waves of 32x32.
#define GS_BK 128
#define GS_STAGE ((64 + 64) * GS_BK)   // bf16 elements of one stage: A tile, then B tile
#define GS_LOADS 8                     // direct loads per wave and stage

// s_waitcnt operand that waits for all but n vector-memory operations and for nothing else
#define GS_VMCNT(n) (((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))

// Workgroup barrier that orders LDS traffic only: vector-memory operations (the direct loads of
// later stages) stay in flight across it, which __syncthreads would not allow.
__device__ __forceinline__ void gs_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ float gs_sigmoid(float x) { return 1.f / (1.f + expf(-x)); }
__device__ __forceinline__ bf16_t gs_bf16(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// MODE 0: C[out_row[r], :] = A[r, :] B^T + bias.
// MODE 1: the product is the gate pre-activations of an LSTM layer (N = 4H, gate-interleaved
// columns) and the epilogue is the cell update; C, out_row and ldc are not used.
// MODE 2: the product is the predictor projection p of new hypotheses (row r = pair r, stored at
// C[out_row[r], :]); the epilogue also forms the joiner input rows act(e[frame] + p) of the pair's
// frames (Section 3.1), so that the next joiner call needs no kernel of its own for them.
// m_dev not null: the kernel was enqueued before the host knew the number of rows.  M is then only
// an upper bound (it sizes the grid and keeps every address inside the buffers); the rows that
// exist are the first *m_dev, read from device memory: workgroups beyond them leave at once, and the
// epilogue stores nothing for the others' surplus rows.
template <int MODE>
__global__ void __launch_bounds__(256)
k_gemm_small(const bf16_t *__restrict__ A, const bf16_t *__restrict__ B, const float *__restrict__ bias,
             float *__restrict__ C, int M, int N, int K, const int *__restrict__ out_row, long ldc, int tiles_m,
             int tiles_n, int ns, LstmEp ep, JoinEp jp, const int *__restrict__ m_dev,
             const int *__restrict__ any_dev, PartEp pe) {
    constexpr bool LSTM = MODE == 1;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];   // ns stages
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    // The 8 XCDs (workgroup id modulo 8) form a 2 x 4 grid over the tiles, so that each XCD's L2
    // fetches half of A and a quarter of B instead of all of both.
    // (MODE 2 may run several workgroups per tile, see JoinEp: the grid is then that many copies of the
    // tile grid, one behind the other)
    const int tmx = (tiles_m + 1) >> 1, tnx = (tiles_n + 3) >> 2;
    const int base_grid = 8 * tmx * tnx;
    const int fgroup = MODE == 2 ? (int)blockIdx.x / base_grid : 0;
    const int bid = MODE == 2 ? (int)blockIdx.x - fgroup * base_grid : (int)blockIdx.x;
    const int xcd = bid & 7, j = bid >> 3;
    int tile_m = (xcd >> 2) * tmx + j % tmx, tile_n = (xcd & 3) * tnx + j / tmx;
    if ((MODE == 0 || MODE == 3) && pe.xcd_rows != 0) {   // a row range per XCD, all its columns
        const int tpx = (tiles_m + 7) >> 3;
        tile_m = xcd * tpx + j % tpx;
        tile_n = j / tpx;
    }
    if (tile_m >= tiles_m || tile_n >= tiles_n) return;   // before any barrier
    const int kt = K / GS_BK;

    // Direct loads: one instruction fills 1 KB of LDS = 4 rows of 256 bytes, lane l the 16 bytes
    // at row l/16, position l%16; the position holds global chunk (l%16) ^ (row & 15).
    const int lrow = lane >> 4, lpos = lane & 15;
    const bf16_t *ga[4], *gb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = i * 16 + wave * 4 + lrow;
        const int ch = (lpos ^ (row & 15)) * 8;
        ga[i] = A + (long)min(tile_m * 64 + row, M - 1) * K + ch;
        gb[i] = B + (long)min(tile_n * 64 + row, N - 1) * K + ch;
    }
    auto fetch = [&](int chunk, int stage) {
        bf16_t *dst = smem + stage * GS_STAGE + wave * 4 * GS_BK;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ga[i] + chunk * GS_BK),
                                             (__attribute__((address_space(3))) void *)(dst + i * 16 * GS_BK), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gb[i] + chunk * GS_BK),
                                             (__attribute__((address_space(3))) void *)(dst + (64 + i * 16) * GS_BK), 16, 0, 0);
    };
    // What the epilogue needs from memory (destination rows, bias) is requested first: loads retire
    // in order, so these are back long before the tiles and cost the epilogue no round trip.
    const int col = tile_n * 64 + wn * 32 + (lane & 31);
    const float bv = (bias && col < N) ? bias[col] : 0.f;
    int orow[16];
    int e_ps = 0, e_ns = 0, e_tok = 0;   // LSTM: the row this lane updates in the epilogue
    int e_f0 = 0;                        // (MODE 2: destination slot, first joiner row, frames, first frame)
    if (LSTM) {
        const int erow = min(tile_m * 64 + wm * 32 + (lane >> 1), M - 1);
        e_ps = ep.pslot[erow];
        e_ns = ep.slot[erow];
        e_tok = ep.tok[erow];   // (unconditionally: a load behind a condition would be waited for at once)
    } else if (MODE == 2) {
        const int erow = min(tile_m * 64 + wm * 32 + (lane >> 1), M - 1);
        e_ns = out_row[erow];
        e_ps = jp.pair_row0[erow];
        e_tok = jp.pair_len[erow];
        e_f0 = jp.pair_frame0[erow];
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = min(tile_m * 64 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3), M - 1);
            orow[r] = out_row ? out_row[row] : row;
        }
    }
    asm volatile("" ::: "memory");
    const int m_live = m_dev ? min(*m_dev, M) : M;   // (the same in every lane: a scalar load)
    if (tile_m * 64 >= m_live) return;   // no row of this tile exists (before anything is on its way into LDS)
    // (slot layout: rows that exist lie anywhere among the M, a dead row has state slot -1; the
    // launch as a whole leaves when the round made no hypothesis at all)
    if (any_dev && *any_dev == 0) return;
    const int first = min(ns, kt);
    for (int c = 0; c < first; ++c) fetch(c, c);
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const int frow = lane & 31, fsel = lane >> 5, fsw = frow & 15;
    const int fa = (wm * 32 + frow) * GS_BK, fb = (64 + wn * 32 + frow) * GS_BK;
    int stage = 0;
    for (int c = 0; c < kt; ++c) {
        // K tiles requested after this one and still allowed to be in flight
        const int after = min(kt, c + ns) - 1 - c;
        if (after >= 3) __builtin_amdgcn_s_waitcnt(GS_VMCNT(3 * GS_LOADS));
        else if (after == 2) __builtin_amdgcn_s_waitcnt(GS_VMCNT(2 * GS_LOADS));
        else if (after == 1) __builtin_amdgcn_s_waitcnt(GS_VMCNT(1 * GS_LOADS));
        else __builtin_amdgcn_s_waitcnt(GS_VMCNT(0));
        gs_barrier();      // every wave's share of this K tile is in LDS
        const bf16_t *cur = smem + stage * GS_STAGE;
        // all fragments of the K tile first, then the matrix instructions back to back
        bf16x8 af[GS_BK / 16], bfr[GS_BK / 16];
#pragma unroll
        for (int kk = 0; kk < GS_BK / 16; ++kk) {
            const int cpos = ((kk * 2 + fsel) ^ fsw) * 8;
            af[kk] = *reinterpret_cast<const bf16x8 *>(cur + fa + cpos);
            bfr[kk] = *reinterpret_cast<const bf16x8 *>(cur + fb + cpos);
        }
#pragma unroll
        for (int kk = 0; kk < GS_BK / 16; ++kk)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk], bfr[kk], acc, 0, 0, 0);
        if (c + ns < kt) {
            gs_barrier();      // every wave has read this stage
            fetch(c + ns, stage);
        }
        stage = stage + 1 == ns ? 0 : stage + 1;
    }
    if (LSTM) {
        // The wave's 32 x 32 block of gates goes through LDS (the stages are free once every wave is
        // past the last K tile) and comes back as 32 rows x 8 hidden units x 4 gates: lane l takes
        // row l/2 and units 4(l%2)..4(l%2)+3, i.e. 16 consecutive floats of the row.
        gs_barrier();
        float *sacc = reinterpret_cast<float *>(smem) + wave * (32 * 36);   // rows padded to 36 floats
#pragma unroll
        for (int r = 0; r < 16; ++r)
            sacc[((r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * 36 + (lane & 31)] = acc[r] + bv;
        const int rowb = lane >> 1, half = lane & 1;
        const int row = tile_m * 64 + wm * 32 + rowb;
        const int j0 = tile_n * 16 + wn * 8 + half * 4;   // first hidden unit of this lane
        float4 g4[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) g4[q] = *reinterpret_cast<const float4 *>(sacc + rowb * 36 + half * 16 + q * 4);
        if (row < m_live && j0 < ep.H && e_ns >= 0) {
            const int H = ep.H;
            // everything the update reads from memory is requested before any of it is used: the
            // parent's cell state, the parent's h of the next layer, the input half of the gates
            // (the latter two from addresses that are valid whether they are needed or not)
            const float4 cp4 = *reinterpret_cast<const float4 *>(ep.c_par + (long)e_ps * H + j0);
            const float4 hp = *reinterpret_cast<const float4 *>((ep.h_par_next ? ep.h_par_next : ep.c_par) + (long)e_ps * H + j0);
            const float4 *eg = ep.emb_gates ? reinterpret_cast<const float4 *>(ep.emb_gates + (long)e_tok * 4 * H + 4 * j0)
                                            : reinterpret_cast<const float4 *>(ep.c_par + (long)e_ps * H + j0);
            const int estep = ep.emb_gates ? 1 : 0;
            float4 e4[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) e4[q] = eg[q * estep];
            if (ep.emb_gates) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    g4[q].x += e4[q].x; g4[q].y += e4[q].y; g4[q].z += e4[q].z; g4[q].w += e4[q].w;
                }
            }
            const float cp[4] = {cp4.x, cp4.y, cp4.z, cp4.w};
            float cn[4], hn[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float ig = gs_sigmoid(g4[q].x), fg = gs_sigmoid(g4[q].y), gg = tanhf(g4[q].z), og = gs_sigmoid(g4[q].w);
                cn[q] = fg * cp[q] + ig * gg;
                hn[q] = og * tanhf(cn[q]);
            }
            *reinterpret_cast<float4 *>(ep.c_new + (long)e_ns * H + j0) = make_float4(cn[0], cn[1], cn[2], cn[3]);
            *reinterpret_cast<float4 *>(ep.h_new + (long)e_ns * H + j0) = make_float4(hn[0], hn[1], hn[2], hn[3]);
            const uint2 hb = make_uint2((unsigned)gs_bf16(hn[0]) | ((unsigned)gs_bf16(hn[1]) << 16),
                                        (unsigned)gs_bf16(hn[2]) | ((unsigned)gs_bf16(hn[3]) << 16));
            if (ep.h_par_next == nullptr) {
                *reinterpret_cast<uint2 *>(ep.out16 + (long)row * H + j0) = hb;
            } else {
                *reinterpret_cast<uint2 *>(ep.out16 + (long)row * 2 * H + j0) = hb;
                *reinterpret_cast<uint2 *>(ep.out16 + (long)row * 2 * H + H + j0) =
                    make_uint2((unsigned)gs_bf16(hp.x) | ((unsigned)gs_bf16(hp.y) << 16),
                               (unsigned)gs_bf16(hp.z) | ((unsigned)gs_bf16(hp.w) << 16));
            }
        }
        return;
    }
    if (MODE == 3) {
        // One-frame segments: no logits leave the kernel.  The tile goes through LDS as above (lane l
        // gets row l/2 of the wave's 32 and 16 consecutive columns), every lane reduces its 16 logits
        // to their maximum, the sum of their exponentials, the blank logit if it is among them and its
        // NP largest non-blank logits, and one thread per row merges the four 16-column pieces of the
        // row into the tile's partial.
        gs_barrier();
        float *sacc = reinterpret_cast<float *>(smem) + wave * (32 * 36);
#pragma unroll
        for (int r = 0; r < 16; ++r)
            sacc[((r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * 36 + (lane & 31)] = acc[r] + bv;
        const int rowb = lane >> 1, half = lane & 1, np = pe.np, pw2 = 3 + 2 * np;
        float q[16];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float4 v = *reinterpret_cast<const float4 *>(sacc + rowb * 36 + half * 16 + k * 4);
            q[4 * k] = v.x; q[4 * k + 1] = v.y; q[4 * k + 2] = v.z; q[4 * k + 3] = v.w;
        }
        const int c0 = tile_n * 64 + wn * 32 + half * 16;
        float mx = -INFINITY, lb = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (c0 + i < N) mx = fmaxf(mx, q[i]);
        float z = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (c0 + i < N) z += __expf(q[i] - mx);
            if (c0 + i == pe.blank) lb = q[i];
            if (c0 + i >= N || c0 + i == pe.blank) q[i] = -INFINITY;   // not a candidate
        }
        if (pe.pieces) {
            // (no second stage: the piece's partial goes out as it is; the reader merges four per tile)
            const int row = tile_m * 64 + wm * 32 + rowb;
            if (row < M) {
                float *out = pe.part + (((long)row * tiles_n + tile_n) * 4 + wn * 2 + half) * part_width(np);
                *reinterpret_cast<float4 *>(out) = make_float4(mx, z, lb, 0.f);
                for (int n = 0; n < np; ++n) {
                    float best = -INFINITY;
                    int bi = -1;
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (q[i] > best) { best = q[i]; bi = i; }   // (ascending columns: the smaller token wins a tie)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (i == bi) q[i] = -INFINITY;
                    out[4 + n] = best;
                    out[4 + np + n] = __int_as_float(bi >= 0 ? c0 + bi : -1);
                }
            }
            return;
        }
        float *spart = reinterpret_cast<float *>(smem) + 4 * (32 * 36);   // [64 rows][4 pieces][3 + 2 NP]
        float *dst = spart + ((wm * 32 + rowb) * 4 + wn * 2 + half) * pw2;
        dst[0] = mx;
        dst[1] = z;
        dst[2] = lb;
        for (int n = 0; n < np; ++n) {
            float best = -INFINITY;
            int bi = -1;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (q[i] > best) { best = q[i]; bi = i; }   // (ascending columns: the smaller token wins a tie)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (i == bi) q[i] = -INFINITY;
            dst[3 + n] = best;
            dst[3 + np + n] = __int_as_float(bi >= 0 ? c0 + bi : -1);
        }
        gs_barrier();
        if (tid < 64) {
            const int row = tile_m * 64 + tid;
            if (row < M) {
                const float *src = spart + tid * 4 * pw2;
                float m = -INFINITY, lbm = -INFINITY;
#pragma unroll
                for (int sgm = 0; sgm < 4; ++sgm) {
                    m = fmaxf(m, src[sgm * pw2]);
                    lbm = fmaxf(lbm, src[sgm * pw2 + 2]);
                }
                float zt = 0.f;
#pragma unroll
                for (int sgm = 0; sgm < 4; ++sgm) {
                    const float ms = src[sgm * pw2];
                    if (ms > -INFINITY) zt += src[sgm * pw2 + 1] * __expf(ms - m);
                }
                float *out = pe.part + ((long)row * tiles_n + tile_n) * part_width(np);
                out[0] = m;
                out[1] = zt;
                out[2] = lbm;
                out[3] = 0.f;
                int i0 = 0, i1 = 0, i2 = 0, i3 = 0;   // heads of the four pieces' lists
                for (int n = 0; n < np; ++n) {
                    const float v0 = i0 < np ? src[0 * pw2 + 3 + i0] : -INFINITY;
                    const float v1 = i1 < np ? src[1 * pw2 + 3 + i1] : -INFINITY;
                    const float v2 = i2 < np ? src[2 * pw2 + 3 + i2] : -INFINITY;
                    const float v3 = i3 < np ? src[3 * pw2 + 3 + i3] : -INFINITY;
                    float best = v0;
                    int bs = 0;
                    if (v1 > best) { best = v1; bs = 1; }   // (pieces in column order: the smaller token wins a tie)
                    if (v2 > best) { best = v2; bs = 2; }
                    if (v3 > best) { best = v3; bs = 3; }
                    const int bidx = bs == 0 ? i0 : (bs == 1 ? i1 : (bs == 2 ? i2 : i3));
                    out[4 + n] = best;
                    out[4 + np + n] = best > -INFINITY ? src[bs * pw2 + 3 + np + bidx] : __int_as_float(-1);
                    if (best > -INFINITY) {
                        i0 += bs == 0; i1 += bs == 1; i2 += bs == 2; i3 += bs == 3;
                    }
                }
            }
        }
        return;
    }
    if (MODE == 2) {
        // Same passage through LDS: lane l takes row l/2 and 16 consecutive columns, stores them
        // as the projection and, for each frame of the pair, adds the encoder row and activates.
        // The first four encoder frames are requested before the passage (clamped addresses, valid
        // in every lane) and nothing is stored before they are used, so their round trip runs
        // beside the barrier and the LDS traffic.
        const int rowb = lane >> 1, half = lane & 1;
        const int row = tile_m * 64 + wm * 32 + rowb;
        const int c0 = tile_n * 64 + wn * 32 + half * 16;
        const int len = e_tok;
        const int fgs = jp.fgroups > 1 ? jp.fgroups : 1;   // this workgroup's frames: fgroup, fgroup + fgs, ...
        uint4 ev0[4][2];
        {
            const int c0c = min(c0, N - 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // (a row that does not exist has no descriptor: frame 0 keeps the address valid)
                const long fr = row < m_live ? (long)e_f0 + max(min(fgroup + q * fgs, len - 1), 0) : 0;
                const uint4 *src = reinterpret_cast<const uint4 *>(jp.enc + fr * N + c0c);
                ev0[q][0] = src[0];
                ev0[q][1] = src[1];
            }
        }
        gs_barrier();
        float *sacc = reinterpret_cast<float *>(smem) + wave * (32 * 36);
#pragma unroll
        for (int r = 0; r < 16; ++r)
            sacc[((r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * 36 + (lane & 31)] = acc[r] + bv;
        float4 p4[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) p4[q] = *reinterpret_cast<const float4 *>(sacc + rowb * 36 + half * 16 + q * 4);
        if (row < m_live && c0 < N && e_ns >= 0) {
            const float p[16] = {p4[0].x, p4[0].y, p4[0].z, p4[0].w, p4[1].x, p4[1].y, p4[1].z, p4[1].w,
                                 p4[2].x, p4[2].y, p4[2].z, p4[2].w, p4[3].x, p4[3].y, p4[3].z, p4[3].w};
            for (int i0 = 0; fgroup + i0 * fgs < len; i0 += 4) {
                uint4 ev[4][2];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (i0 == 0) {
                        ev[q][0] = ev0[q][0];
                        ev[q][1] = ev0[q][1];
                    } else {
                        const uint4 *src = reinterpret_cast<const uint4 *>(
                            jp.enc + (long)(e_f0 + min(fgroup + (i0 + q) * fgs, len - 1)) * N + c0);
                        ev[q][0] = src[0];
                        ev[q][1] = src[1];
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int t = fgroup + (i0 + q) * fgs;
                    if (t < len) {
                        const unsigned w[8] = {ev[q][0].x, ev[q][0].y, ev[q][0].z, ev[q][0].w,
                                               ev[q][1].x, ev[q][1].y, ev[q][1].z, ev[q][1].w};
                        unsigned o[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const float lo = tbs_joiner_act(__uint_as_float(w[i] << 16) + p[2 * i], jp.act);
                            const float hi = tbs_joiner_act(__uint_as_float(w[i] & 0xFFFF0000u) + p[2 * i + 1], jp.act);
                            o[i] = (unsigned)gs_bf16(lo) | ((unsigned)gs_bf16(hi) << 16);
                        }
                        uint4 *dstp = reinterpret_cast<uint4 *>(jp.amat + (long)(e_ps + t) * N + c0);
                        dstp[0] = make_uint4(o[0], o[1], o[2], o[3]);
                        dstp[1] = make_uint4(o[4], o[5], o[6], o[7]);
                    }
                }
            }
            if (fgroup == 0) {
                float4 *crow = reinterpret_cast<float4 *>(C + (long)e_ns * ldc + c0);
#pragma unroll
                for (int q = 0; q < 4; ++q) crow[q] = p4[q];
            }
        }
        return;
    }
    // epilogue: lane holds column (lane & 31); accumulator r is row 8*(r/4) + 4*(lane/32) + r%4.
    // Every address is made before the first store, outside any branch: a wait behind a branch
    // would make each store wait for the store before it.
    float *dst[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) dst[r] = C + (long)orow[r] * ldc + col;
#pragma unroll
    for (int r = 0; r < 16; ++r) asm volatile("" : "+v"(dst[r]));
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = tile_m * 64 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (row < m_live && col < N) *dst[r] = acc[r] + bv;
    }
}

// LDS stages k_gemm_small may use on the current device (0 = kernel not usable)
static int gemm_small_stages() {
    static int stages = -1;
    if (stages < 0) {
        stages = 0;
        for (int ns = 5; ns >= 2; --ns)
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_small<0>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)(ns * GS_STAGE * sizeof(bf16_t))) == hipSuccess &&
                hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_small<1>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)(ns * GS_STAGE * sizeof(bf16_t))) == hipSuccess &&
                hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_small<2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)(ns * GS_STAGE * sizeof(bf16_t))) == hipSuccess &&
                hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_small<3>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)(ns * GS_STAGE * sizeof(bf16_t))) == hipSuccess) {
                stages = ns;
                break;
            }
        (void)hipGetLastError();
    }
    return stages;
}

// The *_fits functions say whether the kernel can run the problem and has at most max_tiles tiles of
// 64 x 64: GS_TILES by default (what pays where kernels are sized by the round's rows: beyond one turn
// and a quarter of workgroups on the 256 CUs the persistent kernel's larger tiles do better), more
// where the caller has measured otherwise (the slot layout, whose other savings outweigh a second
// turn).  The launchers themselves take any number of tiles.
static long gs_tiles(int M, int N) { return (long)((M + 63) / 64) * ((N + 63) / 64); }
// More tiles than CUs: two LDS stages a workgroup (refilled as they are read) instead of one per K
// tile, so that two workgroups share a CU and a second turn of workgroups does not start on an idle
// chip (measured on the Librispeech-like shape: 80 utterances 23.4 -> 19.8 ms per decode, 128
// utterances 24.5 -> 21.1).
static bool gs_two_per_cu(int tiles_m, int tiles_n) { return (long)tiles_m * tiles_n > 256; }

bool gemm_small_fits(int M, int N, int K, int max_tiles) {   // what launch_gemm_bf16 sends to k_gemm_small by itself
    return K % GS_BK == 0 && gemm_small_stages() >= 2 && gs_tiles(M, N) <= max_tiles;
}

bool gemm_lstm_fits(int M, int H, int K, int max_tiles) {
    const int ns_max = gemm_small_stages();
    return ns_max >= 2 && H % 4 == 0 && K % GS_BK == 0 && K / GS_BK <= ns_max && gs_tiles(M, 4 * H) <= max_tiles;
}

hipError_t launch_gemm_lstm(hipStream_t st, const bf16_t *A, const bf16_t *Wp, const float *biasp, int M, int K,
                            const LstmEp &ep, const int *m_dev, const int *any_dev) {
    if (M <= 0) return hipSuccess;
    if (!gemm_lstm_fits(M, ep.H, K, INT_MAX)) return hipErrorInvalidValue;
    const int N = 4 * ep.H, tiles_m = (M + 63) / 64, tiles_n = (N + 63) / 64;
    const int ns = gs_two_per_cu(tiles_m, tiles_n) ? 2 : (K / GS_BK < 2 ? 2 : K / GS_BK);
    const int grid = 8 * ((tiles_m + 1) / 2) * ((tiles_n + 3) / 4);
    hipLaunchKernelGGL(k_gemm_small<1>, dim3(grid), dim3(256), ns * GS_STAGE * sizeof(bf16_t), st, A, Wp, biasp,
                       nullptr, M, N, K, nullptr, 0L, tiles_m, tiles_n, ns, ep, JoinEp{}, m_dev, any_dev, PartEp{});
    return hipGetLastError();
}

bool gemm_part_fits(int M, int N, int K, int np, int max_tiles) {
    // (the epilogue's LDS: four 32 x 36 blocks and 64 x 4 lists of 3 + 2 NP values, inside two stages)
    const size_t lds = sizeof(float) * (4 * 32 * 36 + 64 * 4 * (size_t)(3 + 2 * np));
    return K % GS_BK == 0 && gemm_small_stages() >= 2 && gs_tiles(M, N) <= max_tiles && np >= 1 && np <= 16 &&
           lds <= 2 * GS_STAGE * sizeof(bf16_t);
}

hipError_t launch_gemm_part(hipStream_t st, const bf16_t *A, const bf16_t *B, const float *bias, int M, int N, int K,
                            const PartEp &pe) {
    if (M <= 0) return hipSuccess;
    if (!gemm_part_fits(M, N, K, pe.np, INT_MAX) || !pe.part) return hipErrorInvalidValue;
    const int tiles_m = (M + 63) / 64, tiles_n = (N + 63) / 64;
    const int ns_max = gemm_small_stages();
    const int ns = gs_two_per_cu(tiles_m, tiles_n) ? 2 : (K / GS_BK < ns_max ? (K / GS_BK < 2 ? 2 : K / GS_BK) : ns_max);
    const int grid = pe.xcd_rows ? 8 * ((tiles_m + 7) / 8) * tiles_n : 8 * ((tiles_m + 1) / 2) * ((tiles_n + 3) / 4);
    hipLaunchKernelGGL(k_gemm_small<3>, dim3(grid), dim3(256), ns * GS_STAGE * sizeof(bf16_t), st, A, B, bias, nullptr, M,
                       N, K, nullptr, 0L, tiles_m, tiles_n, ns, LstmEp{}, JoinEp{}, nullptr, nullptr, pe);
    return hipGetLastError();
}

bool gemm_join_fits(int M, int N, int K, int max_tiles) {
    const int ns_max = gemm_small_stages();
    return ns_max >= 2 && N % 16 == 0 && K % GS_BK == 0 && K / GS_BK <= ns_max && gs_tiles(M, N) <= max_tiles;
}

hipError_t launch_gemm_join(hipStream_t st, const bf16_t *A, const bf16_t *B, const float *bias, float *C, int M,
                            int N, int K, const int *out_row, long ldc, const JoinEp &jp, const int *m_dev,
                            const int *any_dev) {
    if (M <= 0) return hipSuccess;
    if (!gemm_join_fits(M, N, K, INT_MAX) || !out_row) return hipErrorInvalidValue;
    const int tiles_m = (M + 63) / 64, tiles_n = (N + 63) / 64;
    const int ns = gs_two_per_cu(tiles_m, tiles_n) ? 2 : (K / GS_BK < 2 ? 2 : K / GS_BK);
    const int grid = 8 * ((tiles_m + 1) / 2) * ((tiles_n + 3) / 4) * (jp.fgroups > 1 ? jp.fgroups : 1);
    hipLaunchKernelGGL(k_gemm_small<2>, dim3(grid), dim3(256), ns * GS_STAGE * sizeof(bf16_t), st, A, B, bias, C, M,
                       N, K, out_row, ldc, tiles_m, tiles_n, ns, LstmEp{}, jp, m_dev, any_dev, PartEp{});
    return hipGetLastError();
}

// kernel: 0 = by size (what the decode uses); 1..4 force one (tests run every kernel on every shape):
// 1 = 64x64 tiles, 2 = 128x128, 3 = 256x256 (all k_gemm_bf16), 4 = k_gemm_small
hipError_t launch_gemm_bf16(hipStream_t st, const bf16_t *A, const bf16_t *B, const float *bias, float *C, int M,
                            int N, int K, const int *out_row, long ldc, int kernel, const int *m_dev, bool xcd_rows) {
    if (M <= 0) return hipSuccess;
    if (m_dev && !gemm_small_fits(M, N, K, INT_MAX)) return hipErrorInvalidValue;   // only k_gemm_small reads its row count
    if ((kernel == 0 || kernel == 4) && K % GS_BK == 0) {
        const int tiles_m = (M + 63) / 64, tiles_n = (N + 63) / 64;
        const int ns_max = gemm_small_stages();
        if (ns_max >= 2 && ((long)tiles_m * tiles_n <= GS_TILES || kernel == 4 || m_dev)) {
            const int ns = gs_two_per_cu(tiles_m, tiles_n) ? 2 : (K / GS_BK < ns_max ? (K / GS_BK < 2 ? 2 : K / GS_BK) : ns_max);
            const int grid = xcd_rows ? 8 * ((tiles_m + 7) / 8) * tiles_n : 8 * ((tiles_m + 1) / 2) * ((tiles_n + 3) / 4);
            PartEp pe{};
            pe.xcd_rows = xcd_rows ? 1 : 0;
            hipLaunchKernelGGL(k_gemm_small<0>, dim3(grid), dim3(256), ns * GS_STAGE * sizeof(bf16_t), st, A, B, bias, C,
                               M, N, K, out_row, ldc, tiles_m, tiles_n, ns, LstmEp{}, JoinEp{}, m_dev, nullptr, pe);
            return hipGetLastError();
        }
    }
    if (kernel == 4) return hipErrorInvalidValue;   // k_gemm_small needs K in multiples of 128
    if (kernel == 0) {
        // measured on MI355X: 256x256 tiles (8 waves, 128x64 per wave) once they fill the chip 1.5
        // times over, 128x128 (two workgroups per CU) for mid sizes, 64x64 so that small problems
        // still spread over the CUs
        long t256 = (long)((M + 255) / 256) * ((N + 255) / 256);
        long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
        kernel = t256 >= 384 ? 3 : (t128 >= 256 ? 2 : 1);
    }
    switch (kernel) {
        case 1: return gemm_launch<1, 1, 2, 2, 64, 4>(st, A, B, bias, C, M, N, K, out_row, ldc);   // 64x64, 4 waves
        case 2: return gemm_launch<2, 2, 2, 2, 64, 2>(st, A, B, bias, C, M, N, K, out_row, ldc);   // 128x128, 4 waves
        case 3: return gemm_launch<4, 2, 2, 4, 64, 1>(st, A, B, bias, C, M, N, K, out_row, ldc);   // 256x256, 8 waves
        default: return hipErrorInvalidValue;
    }
}

// One piece of a large product: rows [*m_begin, *m_end) of A and C, the two bounds read from device
// memory by the kernel; m_max (at least the piece's rows) sizes the launch.  Persistent kernel only.
hipError_t launch_gemm_bf16_rows(hipStream_t st, const bf16_t *A, const bf16_t *B, const float *bias, float *C,
                                 int m_max, int N, int K, long ldc, const int *m_begin, const int *m_end) {
    if (m_max <= 0) return hipSuccess;
    if (!m_begin || !m_end) return hipErrorInvalidValue;
    const long t256 = (long)((m_max + 255) / 256) * ((N + 255) / 256);
    const long t128 = (long)((m_max + 127) / 128) * ((N + 127) / 128);
    if (t256 >= 384) return gemm_launch<4, 2, 2, 4, 64, 1>(st, A, B, bias, C, m_max, N, K, nullptr, ldc, m_begin, m_end);
    if (t128 >= 256) return gemm_launch<2, 2, 2, 2, 64, 2>(st, A, B, bias, C, m_max, N, K, nullptr, ldc, m_begin, m_end);
    return gemm_launch<1, 1, 2, 2, 64, 4>(st, A, B, bias, C, m_max, N, K, nullptr, ldc, m_begin, m_end);
}
