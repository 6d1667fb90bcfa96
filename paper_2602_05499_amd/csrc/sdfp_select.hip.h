// Token selection of the speculative step: Eq. 1 draws, Eq. 2 acceptance test, Eq. 3 resample, rollback.
#pragma once
#include "sdfp_common.hip.h"

namespace sdfp {

// ---- token selection (Eq. 1 draws, Eq. 2 test, Eq. 3 resample) -----------------------------------------
struct Uni { float u[2 * MAX_K + 2]; };

// block-wide helpers for a 1024-thread workgroup; results broadcast through LDS
__device__ __forceinline__ double block_sum_d(double v, double* sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, W = blockDim.x >> 6;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < W; ++w) s += sh[w];
    return s;
}
__device__ __forceinline__ float block_max_f(float v, double* sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, W = blockDim.x >> 6;
    v = wave_max(v);
    __syncthreads();
    if (lane == 0) sh[wave] = (double)v;
    __syncthreads();
    float s = -INFINITY;
    for (int w = 0; w < W; ++w) s = fmaxf(s, (float)sh[w]);
    return s;
}

// weight of token j under `kind`: 0: p = exp((zp-mp)/T)/Sp ; 1: max(0, p - q)
struct CdfSrc {
    const float *zp, *zq;
    float mp, mq;
    double Sp, Sq, invT;
    int kind;
    __device__ __forceinline__ double w(int j) const {
        double p = exp(((double)zp[j] - (double)mp) * invT) / Sp;
        if (kind == 0) return p;
        double q = exp(((double)zq[j] - (double)mq) * invT) / Sq;
        return fmax(0.0, p - q);
    }
};

// smallest j with w_0 + ... + w_j > u * sum(w); every thread scans a contiguous chunk.  Returns the token in
// all threads; *total_out receives sum(w).
__device__ int block_inv_cdf(const CdfSrc& src, int V, double u, double* sh, double* total_out) {
    const int tid = threadIdx.x, T = blockDim.x;
    const int chunk = (V + T - 1) / T, b = min(V, tid * chunk), e = min(V, b + chunk);
    double s = 0.0;
    for (int j = b; j < e; ++j) s += src.w(j);
    __syncthreads();
    sh[64 + tid] = s;
    __syncthreads();
    __shared__ int s_tok;
    __shared__ double s_total;
    if (tid == 0) {
        double tot = 0.0;
        for (int t = 0; t < T; ++t) tot += sh[64 + t];
        s_total = tot;
        const double target = u * tot;
        double run = 0.0;
        int owner = -1;
        for (int t = 0; t < T; ++t) {
            if (run + sh[64 + t] > target) { owner = t; break; }
            run += sh[64 + t];
        }
        s_tok = -1 - owner;            // encode the owning thread; run-before-owner goes to sh[0]
        sh[0] = run;
        sh[1] = target;
    }
    __syncthreads();
    const int owner = -1 - s_tok;
    __syncthreads();
    if (owner < 0) {                   // no crossing (round-off): last index, as min(j, V-1)
        if (tid == 0) s_tok = V - 1;
    } else if (tid == owner) {
        double run = sh[0];
        const double target = sh[1];
        int tok = e - 1;
        for (int j = b; j < e; ++j) {
            run += src.w(j);
            if (run > target) { tok = j; break; }
        }
        s_tok = tok;
    }
    __syncthreads();
    *total_out = s_total;
    return s_tok;
}

__device__ __forceinline__ void row_stats(const float* z, int V, double invT, double* sh, float* mx_out,
                                          double* sum_out) {
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < V; j += blockDim.x) mx = fmaxf(mx, z[j]);
    mx = block_max_f(mx, sh);
    double s = 0.0;
    for (int j = threadIdx.x; j < V; j += blockDim.x) s += exp(((double)z[j] - (double)mx) * invT);
    *sum_out = block_sum_d(s, sh);
    *mx_out = mx;
}

// draw one token from soft-max(z / T) by inverse CDF: draft draws (Eq. 1) and the prefill's first token
__global__ __launch_bounds__(1024) void k_pick_sample(const float* __restrict__ z, int V, float temperature, float u,
                                                      DevState* st, int dst, int off) {
    __shared__ double sh[64 + 1024];
    CdfSrc src;
    src.zp = z; src.zq = nullptr; src.kind = 0; src.invT = 1.0 / (double)temperature;
    row_stats(z, V, src.invT, sh, &src.mp, &src.Sp);
    src.mq = 0.f; src.Sq = 1.0;
    double tot;
    int tok = block_inv_cdf(src, V, (double)u, sh, &tot);
    if (threadIdx.x == 0) {
        if (dst == ROWS_DRAFT) st->d[off] = tok;
        else st->amax[off] = tok;
    }
}

__device__ __forceinline__ void commit_tokens(DevState* st, int* out_tokens, int n, int x, int K) {
    for (int i = 0; i <= n; ++i) {
        const int t = (i < n) ? st->d[i] : x;
        if (st->n_out < st->max_out) out_tokens[st->n_out++] = t;
        else st->overflow = 1;
    }
    st->n_acc = n; st->x = x;
    st->steps += 1; st->drafted += K; st->accepted += n; st->examined += n + (n < K ? 1 : 0);
}

// greedy accept: n = first i with d[i] != arg-max of target row i (else K); x = arg-max of row n
__global__ void k_accept_greedy(DevState* st, int* out_tokens) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int K = st->K;
    int n = K;
    for (int i = 0; i < K; ++i)
        if (st->d[i] != st->amax[i]) { n = i; break; }
    commit_tokens(st, out_tokens, n, st->amax[n], K);
}

// sampling accept: Eq. 2 test per draft token, then Eq. 3 resample or the bonus draw from p_K
__global__ __launch_bounds__(1024) void k_accept_sample(const float* __restrict__ zq, const float* __restrict__ zp,
                                                        int V, float temperature, Uni un, DevState* st,
                                                        int* out_tokens) {
    __shared__ double sh[64 + 1024];
    __shared__ int s_n;
    const int K = st->K;
    const double invT = 1.0 / (double)temperature;
    int n = K;
    for (int i = 0; i < K; ++i) {          // uniform control flow: every thread sees the same decisions
        float mp, mq; double Sp, Sq;
        row_stats(zp + (size_t)i * V, V, invT, sh, &mp, &Sp);
        row_stats(zq + (size_t)i * V, V, invT, sh, &mq, &Sq);
        if (threadIdx.x == 0) {
            const int t = st->d[i];
            const double p = exp(((double)zp[(size_t)i * V + t] - (double)mp) * invT) / Sp;
            const double q = exp(((double)zq[(size_t)i * V + t] - (double)mq) * invT) / Sq;
            s_n = ((double)un.u[i] * q < p) ? 1 : 0;
        }
        __syncthreads();
        const int ok = s_n;
        __syncthreads();
        if (!ok) { n = i; break; }
    }
    CdfSrc src;
    src.invT = invT; src.zp = zp + (size_t)n * V; src.zq = nullptr; src.kind = 0; src.mq = 0.f; src.Sq = 1.0;
    row_stats(src.zp, V, invT, sh, &src.mp, &src.Sp);
    int x;
    double tot;
    if (n < K) {
        src.zq = zq + (size_t)n * V; src.kind = 1;
        row_stats(src.zq, V, invT, sh, &src.mq, &src.Sq);
        x = block_inv_cdf(src, V, (double)un.u[K], sh, &tot);
        if (!(tot > 0.0)) {                 // p == q to the last bit: fall back to p
            src.kind = 0;
            x = block_inv_cdf(src, V, (double)un.u[K], sh, &tot);
        }
    } else {
        x = block_inv_cdf(src, V, (double)un.u[K], sh, &tot);
    }
    if (threadIdx.x == 0) commit_tokens(st, out_tokens, n, x, K);
}

// in-place KV rollback: keep the pending token's and the n accepted drafts' entries
__global__ void k_rollback(DevState* st) {
    if (threadIdx.x == 0 && blockIdx.x == 0) { st->P += st->n_acc + 1; st->t_last = st->x; }
}

// after the prompt forward: commit the first generated token
__global__ void k_commit_first(DevState* st, int* out_tokens, int n_prompt) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        st->P = n_prompt; st->t_last = st->amax[0]; st->n_out = 1; out_tokens[0] = st->amax[0];
        st->n_acc = 0; st->x = st->amax[0]; st->K = 0; st->overflow = 0;
        st->steps = 0; st->drafted = 0; st->accepted = 0; st->examined = 0;
    }
}
__global__ void k_set_k(DevState* st, int K) {
    if (threadIdx.x == 0 && blockIdx.x == 0) st->K = K;
}
__global__ void k_set_pending(DevState* st, int P, int tok) {
    if (threadIdx.x == 0 && blockIdx.x == 0) { st->P = P; st->t_last = tok; }
}
struct DraftBlock { int d[MAX_K]; };
__global__ void k_set_draft(DevState* st, DraftBlock b, int K) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        for (int i = 0; i < K; ++i) st->d[i] = b.d[i];
        st->K = K;
    }
}
__global__ void k_zero_u32(unsigned* p, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0u;
}

}  // namespace sdfp
