// Joiner of token-wise RNN-T beam search: for every live (utterance,
// hypothesis, frame) row r, logits[r, :] = W_out * act(e[frame] + p[hyp]) + b_out
// (Section 3.1: j(t,u,k) = joiner(h, g); Algorithm 1 batches it over the S
// frames of a segment and all hypotheses).  It is a dense contraction
// [rows, Dj] x [Dj, V], so it runs on the matrix cores: the activation rows are
// formed once (add, tanh/relu, round to bf16) and the product is a bf16 MFMA
// GEMM with fp32 accumulation whose epilogue adds the bias and stores the
// logits once.  The same GEMM serves the LSTM gates and the predictor
// projection.  A plain fp32 path exists for fp32 models.
#include "tbs_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

__device__ __forceinline__ bf16_t f2bf(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest, ties to even
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((unsigned)b) << 16); }

__device__ __forceinline__ float joiner_act(float x, int act) { return act == 0 ? tanhf(x) : fmaxf(x, 0.f); }

// ------------------------------------------------------------------ activation rows
// a[r, :] = act(e[row_enc[r], :] + p[row_slot[r], :]), 8 elements per thread.
// (rows_dev: when not null the row count is read from device memory and `rows` only sized the
// grid: the host enqueues the kernel before it knows the count)
__global__ void k_joiner_prep_bf16(int rows, int Dj, int act, const bf16_t *__restrict__ enc,
                                   const float *__restrict__ pool_p, const int *__restrict__ row_enc,
                                   const int *__restrict__ row_slot, bf16_t *__restrict__ amat,
                                   const int *__restrict__ rows_dev, const int *__restrict__ row_begin) {
    // (row_begin not null: the rows [*row_begin, *rows_dev) only, one piece of a large call)
    const int r0 = row_begin ? *row_begin : 0;
    if (rows_dev) rows = *rows_dev;
    int chunks = Dj / 8;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x + (long)r0 * chunks;
    if (idx >= (long)rows * chunks) return;
    int r = (int)(idx / chunks), c = (int)(idx % chunks);
    const uint4 ev = *reinterpret_cast<const uint4 *>(enc + (long)row_enc[r] * Dj + c * 8);
    const float4 p0 = *reinterpret_cast<const float4 *>(pool_p + (long)row_slot[r] * Dj + c * 8);
    const float4 p1 = *reinterpret_cast<const float4 *>(pool_p + (long)row_slot[r] * Dj + c * 8 + 4);
    float e[8] = {__uint_as_float(ev.x << 16), __uint_as_float(ev.x & 0xFFFF0000u),
                  __uint_as_float(ev.y << 16), __uint_as_float(ev.y & 0xFFFF0000u),
                  __uint_as_float(ev.z << 16), __uint_as_float(ev.z & 0xFFFF0000u),
                  __uint_as_float(ev.w << 16), __uint_as_float(ev.w & 0xFFFF0000u)};
    float p[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
    unsigned o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        unsigned lo = f2bf(tbs_joiner_act(e[2 * i] + p[2 * i], act));
        unsigned hi = f2bf(tbs_joiner_act(e[2 * i + 1] + p[2 * i + 1], act));
        o[i] = lo | (hi << 16);
    }
    *reinterpret_cast<uint4 *>(amat + (long)r * Dj + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

// The same by pairs: a thread takes 8 columns of all frames of one (utterance, hypothesis) pair, so the
// pair's p values are read once and its S' frame values are all requested before the first is used.
// (pairs_dev: the number of pairs, in device memory; the grid is sized for the most there can be)
#define PREP_FRAMES 8
__global__ void k_joiner_prep_pairs(int Dj, int act, const bf16_t *__restrict__ enc, const float *__restrict__ pool_p,
                                    const int *__restrict__ pair_row0, const int *__restrict__ pair_len,
                                    const int *__restrict__ pair_frame0, const int *__restrict__ pair_slot,
                                    bf16_t *__restrict__ amat, const int *__restrict__ pairs_dev) {
    const int chunks = Dj / 8;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int j = (int)(idx / chunks), c = (int)(idx - (long)j * chunks);
    if (j >= *pairs_dev) return;
    const int len = pair_len[j];
    const long r0 = pair_row0[j], f0 = pair_frame0[j], slot = pair_slot[j];
    const float4 p0 = *reinterpret_cast<const float4 *>(pool_p + slot * Dj + c * 8);
    const float4 p1 = *reinterpret_cast<const float4 *>(pool_p + slot * Dj + c * 8 + 4);
    const float p[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
    for (int t0 = 0; t0 < len; t0 += PREP_FRAMES) {
        uint4 ev[PREP_FRAMES];
#pragma unroll
        for (int q = 0; q < PREP_FRAMES; ++q)
            ev[q] = *reinterpret_cast<const uint4 *>(enc + (f0 + min(t0 + q, len - 1)) * Dj + c * 8);
#pragma unroll
        for (int q = 0; q < PREP_FRAMES; ++q) {
            if (t0 + q >= len) continue;
            const unsigned w[4] = {ev[q].x, ev[q].y, ev[q].z, ev[q].w};
            unsigned o[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned lo = f2bf(tbs_joiner_act(__uint_as_float(w[i] << 16) + p[2 * i], act));
                const unsigned hi = f2bf(tbs_joiner_act(__uint_as_float(w[i] & 0xFFFF0000u) + p[2 * i + 1], act));
                o[i] = lo | (hi << 16);
            }
            *reinterpret_cast<uint4 *>(amat + (r0 + t0 + q) * Dj + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

hipError_t launch_joiner_prep_pairs(hipStream_t st, const Dims &d, int act, const bf16_t *enc, const float *pool_p,
                                    RowView rv, bf16_t *amat) {
    const long n = (long)d.U * d.N * (d.Dj / 8);
    hipLaunchKernelGGL(k_joiner_prep_pairs, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d.Dj, act, enc, pool_p,
                       rv.pair_row0, rv.pair_len, rv.pair_frame0, rv.pair_slot, amat, rv.counts + TBS_CNT_PAIRS);
    return hipGetLastError();
}

// The same in the slot layout (pair j owns the rows j*S .. j*S + S - 1 and uses the first
// pair_len[j] of them): a row's frame and state slot come from its pair's descriptor.
__global__ void k_joiner_prep_fixed(int rows, int Dj, int S, int act, const bf16_t *__restrict__ enc,
                                    const float *__restrict__ pool_p, const int *__restrict__ pair_len,
                                    const int *__restrict__ pair_frame0, const int *__restrict__ pair_slot,
                                    bf16_t *__restrict__ amat) {
    const int chunks = Dj / 8;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)rows * chunks) return;
    const int r = (int)(idx / chunks), c = (int)(idx % chunks);
    const int j = r / S, t = r - j * S;
    if (t >= pair_len[j]) return;
    const long fr = pair_frame0[j] + t, slot = pair_slot[j];
    const uint4 ev = *reinterpret_cast<const uint4 *>(enc + fr * Dj + c * 8);
    const float4 p0 = *reinterpret_cast<const float4 *>(pool_p + slot * Dj + c * 8);
    const float4 p1 = *reinterpret_cast<const float4 *>(pool_p + slot * Dj + c * 8 + 4);
    const float e[8] = {__uint_as_float(ev.x << 16), __uint_as_float(ev.x & 0xFFFF0000u),
                        __uint_as_float(ev.y << 16), __uint_as_float(ev.y & 0xFFFF0000u),
                        __uint_as_float(ev.z << 16), __uint_as_float(ev.z & 0xFFFF0000u),
                        __uint_as_float(ev.w << 16), __uint_as_float(ev.w & 0xFFFF0000u)};
    const float p[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
    unsigned o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned lo = f2bf(tbs_joiner_act(e[2 * i] + p[2 * i], act));
        const unsigned hi = f2bf(tbs_joiner_act(e[2 * i + 1] + p[2 * i + 1], act));
        o[i] = lo | (hi << 16);
    }
    *reinterpret_cast<uint4 *>(amat + (long)r * Dj + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

hipError_t launch_joiner_prep_fixed(hipStream_t st, const Dims &d, int act, const bf16_t *enc, const float *pool_p,
                                    RowView rv, bf16_t *amat) {
    const int rows = d.U * d.N * d.S;
    const long n = (long)rows * (d.Dj / 8);
    hipLaunchKernelGGL(k_joiner_prep_fixed, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, rows, d.Dj, d.S, act,
                       enc, pool_p, rv.pair_len, rv.pair_frame0, rv.pair_slot, amat);
    return hipGetLastError();
}

__global__ void k_joiner_prep_f32(int rows, int Dj, int act, const float *__restrict__ enc,
                                  const float *__restrict__ pool_p, const int *__restrict__ row_enc,
                                  const int *__restrict__ row_slot, float *__restrict__ amat,
                                  const int *__restrict__ rows_dev) {
    if (rows_dev) rows = *rows_dev;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)rows * Dj) return;
    int r = (int)(idx / Dj), j = (int)(idx % Dj);
    amat[idx] = joiner_act(enc[(long)row_enc[r] * Dj + j] + pool_p[(long)row_slot[r] * Dj + j], act);
}

hipError_t launch_joiner_prep(hipStream_t st, const Dims &d, int dtype, int act, int rows, const void *enc,
                              const float *pool_p, RowView rv, void *amat, const int *rows_dev, const int *row_begin) {
    if (rows <= 0) return hipSuccess;
    if (row_begin && (dtype != 1 || !rows_dev)) return hipErrorInvalidValue;
    if (dtype == 1) {
        long n = (long)rows * (d.Dj / 8);
        hipLaunchKernelGGL(k_joiner_prep_bf16, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, rows, d.Dj, act,
                           (const bf16_t *)enc, pool_p, rv.row_enc, rv.row_slot, (bf16_t *)amat, rows_dev, row_begin);
    } else {
        long n = (long)rows * d.Dj;
        hipLaunchKernelGGL(k_joiner_prep_f32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, rows, d.Dj, act,
                           (const float *)enc, pool_p, rv.row_enc, rv.row_slot, (float *)amat, rows_dev);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ fp32 GEMM (fp32 models)
// C[M,N] = A[M,K] * B[N,K]^T + bias, 64x64 tile, 4x4 outputs per thread.
__global__ void __launch_bounds__(256)
k_gemm_f32(const float *__restrict__ A, const float *__restrict__ B, const float *__restrict__ bias,
           float *__restrict__ C, int M, int N, int K, const int *__restrict__ out_row, long ldc) {
    __shared__ float sA[16][64 + 1], sB[16][64 + 1];
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = tid; i < 64 * 16; i += 256) {
            int r = i / 16, k = i % 16;
            int gm = m0 + r, gn = n0 + r, gk = k0 + k;
            sA[k][r] = (gm < M && gk < K) ? A[(long)gm * K + gk] : 0.f;
            sB[k][r] = (gn < N && gk < K) ? B[(long)gn * K + gk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sA[k][ty * 4 + i]; b[i] = sB[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
        long orow = out_row ? out_row[gm] : gm;
        for (int j = 0; j < 4; ++j) {
            int gn = n0 + tx * 4 + j;
            if (gn < N) C[orow * ldc + gn] = acc[i][j] + (bias ? bias[gn] : 0.f);
        }
    }
}

hipError_t launch_gemm_f32(hipStream_t st, const float *A, const float *B, const float *bias, float *C, int M, int N,
                           int K, const int *out_row, long ldc) {
    if (M <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_gemm_f32, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, st, A, B, bias, C, M, N, K,
                       out_row, ldc);
    return hipGetLastError();
}
