// UpdatePredictorOutput of Algorithm 1: for every hypothesis created in this
// round, run the prediction network one step from its parent's recurrent state
// (Section 3.1: g(u) = predictor(y)).  Embedding lookup and state gather build
// the LSTM input rows, the gate pre-activations are one GEMM against the
// concatenated [W_ih | W_hh] matrix, the cell update is a pointwise kernel, and
// the projection to the joint space is a GEMM that scatters into the state pool.
#include "tbs_internal.h"

__device__ __forceinline__ bf16_t f2bf_p(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float sigmoidf_(float x) { return 1.f / (1.f + expf(-x)); }

// xh[j, :] = [ embed[token_j, 0:E] | h_parent_j(layer 0)[0:H] ]
// (Both gather kernels take the number of pairs from device memory and leave when launched
// beyond it: the host enqueues them on the largest possible grid before it knows the count.)
__global__ void k_pred_gather(Dims d, int dtype, AView A, RowView rv, const void *embed, const float *pool_h,
                              void *xh) {
    int j = blockIdx.x;
    if (j >= rv.counts[TBS_CNT_PAIRS]) return;
    int u = rv.pair_u[j], h = rv.pair_h[j];
    long a = (long)u * d.N + h;
    int tok = A.token[a];
    long ps = A.pslot[a];
    int W = d.E + d.H;
    if (dtype == 1) {
        const bf16_t *em = (const bf16_t *)embed + (long)tok * d.E;
        bf16_t *x = (bf16_t *)xh + (long)j * W;
        for (int i = threadIdx.x; i < d.E; i += blockDim.x) x[i] = em[i];
        for (int i = threadIdx.x; i < d.H; i += blockDim.x) x[d.E + i] = f2bf_p(pool_h[ps * d.H + i]);
    } else {
        const float *em = (const float *)embed + (long)tok * d.E;
        float *x = (float *)xh + (long)j * W;
        for (int i = threadIdx.x; i < d.E; i += blockDim.x) x[i] = em[i];
        for (int i = threadIdx.x; i < d.H; i += blockDim.x) x[d.E + i] = pool_h[ps * d.H + i];
    }
}

hipError_t launch_pred_gather(hipStream_t st, const Dims &d, int dtype, int pairs, AView A, RowView rv,
                              const void *embed, const float *pool_h, void *xh) {
    if (pairs <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_pred_gather, dim3(pairs), dim3(256), 0, st, d, dtype, A, rv, embed, pool_h, xh);
    return hipGetLastError();
}

// bf16 models: the embedding half of the first layer's gates is a table made once
// (embed * W_ih^T + b for every token), so the per-round input is only the parent's h.
__global__ void k_pred_gather_h(Dims d, AView A, RowView rv, const float *pool_h, bf16_t *xh) {
    int j = blockIdx.x;
    if (j >= rv.counts[TBS_CNT_PAIRS]) return;
    long ps = rv.pair_pslot[j];
    bf16_t *x = xh + (long)j * d.H;
    for (int i = threadIdx.x; i < d.H; i += blockDim.x) x[i] = f2bf_p(pool_h[ps * d.H + i]);
}

hipError_t launch_pred_gather_h(hipStream_t st, const Dims &d, int pairs, AView A, RowView rv, const float *pool_h,
                                bf16_t *xh) {
    if (pairs <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_pred_gather_h, dim3(pairs), dim3(256), 0, st, d, A, rv, pool_h, xh);
    return hipGetLastError();
}

// LSTM cell, gate order i, f, g, o; gates already hold W x + W h + b.
__global__ void k_lstm_pointwise(Dims d, int dtype, int layer, AView A, RowView rv, const float *gates,
                                 float *pool_h, float *pool_c, long pool_rows, void *xh_next, void *htop,
                                 const float *emb_gates) {
    int j = blockIdx.x;
    long ps = rv.pair_pslot[j], ns = rv.pair_slot[j];   // parent's and own state slot
    const float *g = gates + (long)j * 4 * d.H;
    // first layer of bf16 models: the embedding half of the gates (and the bias) comes from the table
    const float *eg = emb_gates ? emb_gates + (long)rv.pair_tok[j] * 4 * d.H : nullptr;
    const float *c_par = pool_c + ((long)layer * pool_rows + ps) * d.H;
    float *c_new = pool_c + ((long)layer * pool_rows + ns) * d.H;
    float *h_new = pool_h + ((long)layer * pool_rows + ns) * d.H;
    const bool last = layer + 1 == d.L;
    const float *h_par_next = last ? nullptr : pool_h + ((long)(layer + 1) * pool_rows + ps) * d.H;
    for (int i = threadIdx.x; i < d.H; i += blockDim.x) {
        float gi = g[i], gf = g[d.H + i], gc = g[2 * d.H + i], go = g[3 * d.H + i];
        if (eg) { gi += eg[i]; gf += eg[d.H + i]; gc += eg[2 * d.H + i]; go += eg[3 * d.H + i]; }
        float ig = sigmoidf_(gi);
        float fg = sigmoidf_(gf);
        float gg = tanhf(gc);
        float og = sigmoidf_(go);
        float c = fg * c_par[i] + ig * gg;
        float hv = og * tanhf(c);
        c_new[i] = c;
        h_new[i] = hv;
        if (dtype == 1) {
            if (last) ((bf16_t *)htop)[(long)j * d.H + i] = f2bf_p(hv);
            else {
                bf16_t *x = (bf16_t *)xh_next + (long)j * 2 * d.H;
                x[i] = f2bf_p(hv);
                x[d.H + i] = f2bf_p(h_par_next[i]);
            }
        } else {
            if (last) ((float *)htop)[(long)j * d.H + i] = hv;
            else {
                float *x = (float *)xh_next + (long)j * 2 * d.H;
                x[i] = hv;
                x[d.H + i] = h_par_next[i];
            }
        }
    }
}

hipError_t launch_lstm_pointwise(hipStream_t st, const Dims &d, int dtype, int pairs, int layer, AView A, RowView rv,
                                 const float *gates, float *pool_h, float *pool_c, long pool_rows, void *xh_next,
                                 void *htop, const float *emb_gates) {
    if (pairs <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_lstm_pointwise, dim3(pairs), dim3(256), 0, st, d, dtype, layer, A, rv, gates, pool_h,
                       pool_c, pool_rows, xh_next, htop, emb_gates);
    return hipGetLastError();
}

// wcat[r, :] = [ w_ih[r, 0:in] | w_hh[r, 0:hid] ], elements of 2 bytes
__global__ void k_concat16(const uint16_t *w_ih, const uint16_t *w_hh, uint16_t *wcat, int rows, int in_dim,
                           int hid) {
    long W = in_dim + hid;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * W) return;
    long r = idx / W, c = idx % W;
    wcat[idx] = c < in_dim ? w_ih[r * in_dim + c] : w_hh[r * hid + (c - in_dim)];
}
__global__ void k_concat32(const uint32_t *w_ih, const uint32_t *w_hh, uint32_t *wcat, int rows, int in_dim,
                           int hid) {
    long W = in_dim + hid;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * W) return;
    long r = idx / W, c = idx % W;
    wcat[idx] = c < in_dim ? w_ih[r * in_dim + c] : w_hh[r * hid + (c - in_dim)];
}

hipError_t launch_concat_weights(hipStream_t st, int elem_bytes, const void *w_ih, const void *w_hh, void *wcat,
                                 int rows, int in_dim, int hid) {
    long n = (long)rows * (in_dim + hid);
    unsigned blocks = (unsigned)((n + 255) / 256);
    if (elem_bytes == 2)
        hipLaunchKernelGGL(k_concat16, dim3(blocks), dim3(256), 0, st, (const uint16_t *)w_ih, (const uint16_t *)w_hh,
                           (uint16_t *)wcat, rows, in_dim, hid);
    else
        hipLaunchKernelGGL(k_concat32, dim3(blocks), dim3(256), 0, st, (const uint32_t *)w_ih, (const uint32_t *)w_hh,
                           (uint32_t *)wcat, rows, in_dim, hid);
    return hipGetLastError();
}

// dst row 4j+g = src row g*H+j (rows of row_bytes bytes, a multiple of 4): the gate-interleaved
// order the fused gate GEMM wants
__global__ void k_permute_gate_rows(const uint32_t *src, uint32_t *dst, int H, long row_words) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= 4L * H * row_words) return;
    const long r = idx / row_words, w = idx % row_words;
    const long j = r >> 2, g = r & 3;
    dst[idx] = src[(g * H + j) * row_words + w];
}

hipError_t launch_permute_gate_rows(hipStream_t st, const void *src, void *dst, int H, long row_bytes) {
    const long words = row_bytes / 4, n = 4L * H * words;
    hipLaunchKernelGGL(k_permute_gate_rows, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const uint32_t *)src,
                       (uint32_t *)dst, H, words);
    return hipGetLastError();
}

// ------------------------------------------------------------------ streaming: frame buffer
// Copies whole frames (rows) between the caller's array, the per-utterance frame buffers and
// the spare area used to move leftovers to the front.  UNIT = 16 or 4 bytes.
template <typename UNIT>
__global__ void k_stream_copy(int U, const UNIT *__restrict__ src, UNIT *__restrict__ dst, const int *__restrict__ desc,
                              long row_units) {
    const int u = blockIdx.x;
    const long s0 = (long)desc[u] * row_units, d0 = (long)desc[U + u] * row_units;
    const long total = (long)desc[2 * U + u] * row_units;
    for (long i = (long)blockIdx.y * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.y * blockDim.x)
        dst[d0 + i] = src[s0 + i];
}

hipError_t launch_stream_copy(hipStream_t st, int U, const void *src, void *dst, const int *desc, long row_bytes) {
    if (U <= 0) return hipSuccess;
    const bool wide = row_bytes % 16 == 0 && (reinterpret_cast<uintptr_t>(src) & 15) == 0 &&
                      (reinterpret_cast<uintptr_t>(dst) & 15) == 0;
    const dim3 grid(U, 4), block(256);
    if (wide)
        hipLaunchKernelGGL(k_stream_copy<uint4>, grid, block, 0, st, U, (const uint4 *)src, (uint4 *)dst, desc,
                           row_bytes / 16);
    else
        hipLaunchKernelGGL(k_stream_copy<unsigned>, grid, block, 0, st, U, (const unsigned *)src, (unsigned *)dst, desc,
                           row_bytes / 4);
    return hipGetLastError();
}

// ------------------------------------------------------------------ timing yardstick
__global__ void k_empty() {}
hipError_t launch_empty(hipStream_t st) {
    hipLaunchKernelGGL(k_empty, dim3(1), dim3(64), 0, st);
    return hipGetLastError();
}
