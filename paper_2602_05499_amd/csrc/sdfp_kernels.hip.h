// Device code of libsdfp for gfx950 (CDNA4, wave64): the phases of one transformer forward of M <= 9 rows
// over a contiguous KV cache, plus the token-selection kernels of the speculative step
// (paper Sec. II-A Eq. 1-3, Alg. 1 Stage B).
//
// Precision contract: weight matrices and KV entries are stored as float32 or bfloat16; every activation,
// accumulator and logit is float32.  Every output row's arithmetic (order of every sum) is independent of
// how many rows M share the launch, so row i of a (K+1)-row verify forward is bit-identical to the one-row
// decode of the same prefix: this is what makes greedy speculative output equal plain decoding exactly.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sdfp {

typedef unsigned short bf16_t;   // raw bfloat16 bits
constexpr int MAX_K = 8;
constexpr int MAX_ROWS = MAX_K + 1;
constexpr int ATT_SL = 128;      // attention split length in positions (fixed absolute boundaries)
constexpr int ATT_QC = 16;       // query vectors processed per pass inside an attention workgroup

// ---- device-resident decode state: written by kernels, read by the next call without host round trips ---
struct DevState {
    int P;          // cache_len: positions held in the KV cache
    int t_last;     // pending token
    int n_acc;      // accepted draft tokens of the last step
    int x;          // extra target-derived token of the last step
    int K;          // speculation depth of the current step
    int n_out;      // committed tokens in the output list
    int max_out;
    int overflow;   // set if the output list was full
    long long steps, drafted, accepted, examined;
    int d[MAX_K];           // draft block
    int amax[MAX_ROWS];     // arg-max of each verify row
    int pad[3];
};

// Which tokens / positions the rows of a forward hold.
enum { ROWS_PROMPT = 0, ROWS_DRAFT = 1, ROWS_VERIFY = 2 };
struct Rows {
    int M;     // number of rows
    int src;   // ROWS_*
    int off;   // ROWS_PROMPT: absolute position of row 0; ROWS_DRAFT: draft index i (row sits at P + i)
};

__device__ __forceinline__ int row_pos(const Rows& r, const DevState* st, int m) {
    if (r.src == ROWS_PROMPT) return r.off + m;
    if (r.src == ROWS_DRAFT) return st->P + r.off;
    return st->P + m;
}
__device__ __forceinline__ int row_tok(const Rows& r, const DevState* st, const int* prompt, int m) {
    if (r.src == ROWS_PROMPT) return prompt[r.off + m];
    int i = (r.src == ROWS_DRAFT) ? r.off : m;
    return i == 0 ? st->t_last : st->d[i - 1];
}

// ---- storage types -------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((unsigned)b) << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {   // round-to-nearest-even, finite inputs
    unsigned u = __float_as_uint(f);
    return (bf16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
template <typename WT> struct ST;
template <> struct ST<float> {
    static constexpr int VEC = 4;   // elements per 16-byte load
    static __device__ __forceinline__ float ld(const float* p) { return *p; }
    static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
    static __device__ __forceinline__ void unpack(const uint4& r, float (&w)[4]) {
        w[0] = __uint_as_float(r.x); w[1] = __uint_as_float(r.y);
        w[2] = __uint_as_float(r.z); w[3] = __uint_as_float(r.w);
    }
};
template <> struct ST<bf16_t> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
    static __device__ __forceinline__ void unpack(const uint4& r, float (&w)[8]) {
        w[0] = __uint_as_float(r.x << 16); w[1] = __uint_as_float(r.x & 0xFFFF0000u);
        w[2] = __uint_as_float(r.y << 16); w[3] = __uint_as_float(r.y & 0xFFFF0000u);
        w[4] = __uint_as_float(r.z << 16); w[5] = __uint_as_float(r.z & 0xFFFF0000u);
        w[6] = __uint_as_float(r.w << 16); w[7] = __uint_as_float(r.w & 0xFFFF0000u);
    }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

// ---- a1: embedding gather ------------------------------------------------------------------------------
template <typename WT>
__global__ void k_embed(const WT* __restrict__ emb, float* __restrict__ h, int d, Rows rows, const DevState* st,
                        const int* __restrict__ prompt) {
    int m = blockIdx.y;
    if (m >= rows.M) return;
    int tok = row_tok(rows, st, prompt, m);
    const WT* e = emb + (size_t)tok * d;
    for (int k = blockIdx.x * blockDim.x + threadIdx.x; k < d; k += gridDim.x * blockDim.x)
        h[(size_t)m * d + k] = ST<WT>::ld(e + k);
}

// ---- weight-streaming skinny GEMM core -----------------------------------------------------------------
// Y[m][n] = sum_k W[n][k] * X[m][k] for M <= MT rows.  One wave owns R weight rows for the whole K range;
// lanes split K in 16-byte pieces (coalesced HBM reads); X is staged through LDS in K-tiles (optionally
// RMS-normalised on the way in); accumulation is float32 in a fixed order that does not depend on M.
template <typename WT> struct Tile {
    static constexpr int IT = 4;                          // 16-byte loads per lane per row per tile
    static constexpr int KT = 64 * ST<WT>::VEC * IT;      // K-tile length (bf16 2048, f32 1024)
};

// Op concept:  void wrows(int item, const WT* (&r)[R]) const;  void done(int item, float (&acc)[R][MT], int lane);
template <typename WT, int MT, int R, class Op>
__device__ __forceinline__ void gemv_phase(Op& op, int n_items, const float* __restrict__ xsrc, int M, int Kd,
                                           const float* __restrict__ gain, float eps, float* xs, float* red,
                                           int wg, int n_wg) {
    constexpr int VEC = ST<WT>::VEC, IT = Tile<WT>::IT, KT = Tile<WT>::KT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, W = blockDim.x >> 6;
    float* rs = red + MT * 16;   // [MT] reciprocal RMS per row (1 when no norm)

    if (gain != nullptr) {       // RMSNorm prologue: rs[m] = 1 / sqrt(mean(x_m^2) + eps)
        for (int m = 0; m < M; ++m) {
            float s = 0.f;
            for (int k = tid; k < Kd; k += blockDim.x) {
                float v = xsrc[(size_t)m * Kd + k];
                s = fmaf(v, v, s);
            }
            s = wave_sum(s);
            if (lane == 0) red[m * 16 + wave] = s;
        }
        __syncthreads();
        if (tid < M) {
            float s = 0.f;
            for (int w = 0; w < W; ++w) s += red[tid * 16 + w];
            rs[tid] = 1.0f / sqrtf(s / (float)Kd + eps);
        }
        __syncthreads();
    }

    for (int batch = wg; batch * W < n_items; batch += n_wg) {
        const int item = batch * W + wave;
        const bool active = item < n_items;
        const WT* wr[R];
        if (active) op.wrows(item, wr);
        else
            for (int r = 0; r < R; ++r) wr[r] = nullptr;
        float acc[R][MT];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[r][m] = 0.f;

        uint4 raw[IT][R];
        // prefetch the first tile's weights
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            int k = (it * 64 + lane) * VEC;
#pragma unroll
            for (int r = 0; r < R; ++r)
                raw[it][r] = (active && k < Kd) ? *reinterpret_cast<const uint4*>(wr[r] + k) : make_uint4(0, 0, 0, 0);
        }
        for (int k0 = 0; k0 < Kd; k0 += KT) {
            const int klen = min(KT, Kd - k0);
            __syncthreads();   // everyone finished reading the previous tile
            for (int idx = tid * 4; idx < MT * klen; idx += blockDim.x * 4) {
                int m = idx / klen, kk = idx - m * klen;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (m < M) {
                    v = *reinterpret_cast<const float4*>(xsrc + (size_t)m * Kd + k0 + kk);
                    if (gain != nullptr) {
                        float4 g = *reinterpret_cast<const float4*>(gain + k0 + kk);
                        float r = rs[m];
                        v.x = v.x * r * g.x; v.y = v.y * r * g.y; v.z = v.z * r * g.z; v.w = v.w * r * g.w;
                    }
                }
                *reinterpret_cast<float4*>(xs + m * KT + kk) = v;
            }
            __syncthreads();
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int kk = (it * 64 + lane) * VEC;
                uint4 cur[R];
#pragma unroll
                for (int r = 0; r < R; ++r) cur[r] = raw[it][r];
                // refill this slot with the next tile's weights before computing
                const int kn = k0 + KT + kk;
#pragma unroll
                for (int r = 0; r < R; ++r)
                    raw[it][r] = (active && kn < Kd) ? *reinterpret_cast<const uint4*>(wr[r] + kn) : make_uint4(0, 0, 0, 0);
                if (kk < klen) {
                    float wf[R][VEC];
#pragma unroll
                    for (int r = 0; r < R; ++r) ST<WT>::unpack(cur[r], wf[r]);
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        float xv[VEC];
#pragma unroll
                        for (int v4 = 0; v4 < VEC; v4 += 4) {
                            float4 t = *reinterpret_cast<const float4*>(xs + m * KT + kk + v4);
                            xv[v4] = t.x; xv[v4 + 1] = t.y; xv[v4 + 2] = t.z; xv[v4 + 3] = t.w;
                        }
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int v = 0; v < VEC; ++v) acc[r][m] = fmaf(wf[r][v], xv[v], acc[r][m]);
                    }
                }
            }
        }
        if (active) {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int m = 0; m < MT; ++m) acc[r][m] = wave_sum(acc[r][m]);
            op.done(item, acc, lane);
        }
    }
}

// LDS needed by gemv_phase, in floats
template <typename WT, int MT> constexpr int gemv_lds_floats() { return MT * Tile<WT>::KT + MT * 16 + MT + 3; }

struct LayerDims {
    int d, H, Hkv, hd, F, V, max_seq;
};

// ---- a2: RMSNorm -> QKV projection -> RoPE -> KV append ------------------------------------------------
// Work item = 4 rows of one head: dims (i, i+1, i+hd/2, i+hd/2+1), so each rotary pair sits in one wave.
template <typename WT, int MT>
struct QkvOp {
    const WT *wq, *wk, *wv;
    WT *kc, *vc;             // this layer's K and V cache planes [Hkv][max_seq][hd]
    float* q;                // [M][H*hd]
    const float *cosT, *sinT;  // [max_seq][hd/2]
    LayerDims L;
    Rows rows;
    const DevState* st;
    __device__ __forceinline__ void wrows(int item, const WT* (&r)[4]) const {
        const int per = L.hd >> 2, hs = item / per, i = (item - hs * per) * 2, half = L.hd >> 1;
        const WT* base;
        if (hs < L.H) base = wq + (size_t)hs * L.hd * L.d;
        else if (hs < L.H + L.Hkv) base = wk + (size_t)(hs - L.H) * L.hd * L.d;
        else base = wv + (size_t)(hs - L.H - L.Hkv) * L.hd * L.d;
        r[0] = base + (size_t)i * L.d; r[1] = base + (size_t)(i + 1) * L.d;
        r[2] = base + (size_t)(i + half) * L.d; r[3] = base + (size_t)(i + half + 1) * L.d;
    }
    __device__ __forceinline__ void done(int item, float (&acc)[4][MT], int lane) const {
        const int per = L.hd >> 2, hs = item / per, i = (item - hs * per) * 2, half = L.hd >> 1;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            if (lane == m && m < rows.M) {
                const int pos = row_pos(rows, st, m);
                float a0 = acc[0][m], a1 = acc[1][m], b0 = acc[2][m], b1 = acc[3][m];
                if (hs < L.H + L.Hkv) {   // rotary: (a, b) -> (a cos - b sin, b cos + a sin)
                    const float c0 = cosT[(size_t)pos * half + i], s0 = sinT[(size_t)pos * half + i];
                    const float c1 = cosT[(size_t)pos * half + i + 1], s1 = sinT[(size_t)pos * half + i + 1];
                    float ra0 = a0 * c0 - b0 * s0, rb0 = b0 * c0 + a0 * s0;
                    float ra1 = a1 * c1 - b1 * s1, rb1 = b1 * c1 + a1 * s1;
                    a0 = ra0; b0 = rb0; a1 = ra1; b1 = rb1;
                }
                if (hs < L.H) {
                    float* o = q + (size_t)m * L.H * L.hd + (size_t)hs * L.hd;
                    o[i] = a0; o[i + 1] = a1; o[i + half] = b0; o[i + half + 1] = b1;
                } else {
                    const bool isk = hs < L.H + L.Hkv;
                    const int kvh = isk ? hs - L.H : hs - L.H - L.Hkv;
                    WT* o = (isk ? kc : vc) + ((size_t)kvh * L.max_seq + pos) * L.hd;
                    ST<WT>::st(o + i, a0); ST<WT>::st(o + i + 1, a1);
                    ST<WT>::st(o + i + half, b0); ST<WT>::st(o + i + half + 1, b1);
                }
            }
        }
    }
};

template <typename WT, int MT>
__global__ __launch_bounds__(512) void k_qkv(QkvOp<WT, MT> op, const float* __restrict__ h,
                                             const float* __restrict__ gain, float eps) {
    extern __shared__ float lds[];
    float* xs = lds;
    float* red = lds + MT * Tile<WT>::KT;
    const int n_items = (op.L.H + 2 * op.L.Hkv) * (op.L.hd >> 2);
    gemv_phase<WT, MT, 4>(op, n_items, h, op.rows.M, op.L.d, gain, eps, xs, red, blockIdx.x, gridDim.x);
}

// ---- a4 / a6: projection + residual add ----------------------------------------------------------------
template <typename WT, int MT, int R>
struct ResidOp {
    const WT* w;   // [N][Kd]
    float* h;      // [M][N] residual stream, updated in place
    int N, Kd, M;
    __device__ __forceinline__ void wrows(int item, const WT* (&r)[R]) const {
#pragma unroll
        for (int j = 0; j < R; ++j) r[j] = w + (size_t)min(item * R + j, N - 1) * Kd;
    }
    __device__ __forceinline__ void done(int item, float (&acc)[R][MT], int lane) const {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < R; ++j)
                if (lane == m * R + j && m < M && item * R + j < N) h[(size_t)m * N + item * R + j] += acc[j][m];
    }
};

template <typename WT, int MT, int R>
__global__ __launch_bounds__(512) void k_resid(ResidOp<WT, MT, R> op, const float* __restrict__ x) {
    extern __shared__ float lds[];
    const int n_items = (op.N + R - 1) / R;
    gemv_phase<WT, MT, R>(op, n_items, x, op.M, op.Kd, nullptr, 0.f, lds, lds + MT * Tile<WT>::KT, blockIdx.x,
                          gridDim.x);
}

// ---- a5: RMSNorm -> gate/up projection -> SiLU * mul ---------------------------------------------------
template <typename WT, int MT>
struct GateUpOp {
    const WT *wg, *wu;   // [F][d]
    float* a;            // [M][F]
    int F, d, M;
    __device__ __forceinline__ void wrows(int item, const WT* (&r)[4]) const {
        const int j0 = item * 2, j1 = min(j0 + 1, F - 1);
        r[0] = wg + (size_t)j0 * d; r[1] = wg + (size_t)j1 * d;
        r[2] = wu + (size_t)j0 * d; r[3] = wu + (size_t)j1 * d;
    }
    __device__ __forceinline__ void done(int item, float (&acc)[4][MT], int lane) const {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                if (lane == m * 2 + j && m < M && item * 2 + j < F) {
                    const float g = acc[j][m], u = acc[2 + j][m];
                    a[(size_t)m * F + item * 2 + j] = (g / (1.0f + __expf(-g))) * u;
                }
    }
};

template <typename WT, int MT>
__global__ __launch_bounds__(512) void k_gateup(GateUpOp<WT, MT> op, const float* __restrict__ h,
                                                const float* __restrict__ gain, float eps) {
    extern __shared__ float lds[];
    const int n_items = (op.F + 1) / 2;
    gemv_phase<WT, MT, 4>(op, n_items, h, op.M, op.d, gain, eps, lds, lds + MT * Tile<WT>::KT, blockIdx.x, gridDim.x);
}

// ---- a7: final RMSNorm -> output projection -> fused arg-max -------------------------------------------
// Every wave keeps the running (max, lowest index) of the rows it produced; workgroups publish partials and
// the last one to finish reduces them in workgroup order and writes the token(s).
struct HeadOut {
    float* logits;        // [M][V] or nullptr
    float* part_val;      // [gridDim.x][MAX_ROWS]
    int* part_idx;        // [gridDim.x][MAX_ROWS]
    unsigned* counter;    // arrival counter (left at 0)
    int dst;              // ROWS_DRAFT: st->d[off] ; otherwise st->amax[m]
    int off;
};

template <typename WT, int MT>
struct HeadOp {
    const WT* w;   // [V][d]
    int V, d, M;
    float* logits;
    float best_v[MT];
    int best_i[MT];
    __device__ __forceinline__ void wrows(int item, const WT* (&r)[4]) const {
#pragma unroll
        for (int j = 0; j < 4; ++j) r[j] = w + (size_t)min(item * 4 + j, V - 1) * d;
    }
    __device__ __forceinline__ void done(int item, float (&acc)[4][MT], int lane) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = item * 4 + j;
                if (n < V) {
                    const float v = acc[j][m];
                    if (v > best_v[m] || (v == best_v[m] && n < best_i[m])) { best_v[m] = v; best_i[m] = n; }
                    if (logits != nullptr && lane == ((m * 4 + j) & 63) && m < M) logits[(size_t)m * V + n] = v;
                }
            }
    }
};

template <typename WT, int MT>
__global__ __launch_bounds__(512) void k_head(const WT* __restrict__ w, const float* __restrict__ h,
                                              const float* __restrict__ gain, float eps, int V, int d, int M,
                                              HeadOut out, DevState* st) {
    extern __shared__ float lds[];
    float* red = lds + MT * Tile<WT>::KT;
    HeadOp<WT, MT> op;
    op.w = w; op.V = V; op.d = d; op.M = M; op.logits = out.logits;
#pragma unroll
    for (int m = 0; m < MT; ++m) { op.best_v[m] = -INFINITY; op.best_i[m] = 0x7FFFFFFF; }
    gemv_phase<WT, MT, 4>(op, (V + 3) / 4, h, M, d, gain, eps, lds, red, blockIdx.x, gridDim.x);

    // workgroup reduce of the per-wave bests (wave order, lowest index wins ties)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, W = blockDim.x >> 6;
    __syncthreads();
    float* sv = lds;                                        // [W][MT]
    int* si = reinterpret_cast<int*>(lds + 16 * MT);        // [W][MT]
    if (lane == 0)
#pragma unroll
        for (int m = 0; m < MT; ++m) { sv[wave * MT + m] = op.best_v[m]; si[wave * MT + m] = op.best_i[m]; }
    __syncthreads();
    if (tid < M) {
        float bv = -INFINITY; int bi = 0x7FFFFFFF;
        for (int w2 = 0; w2 < W; ++w2) {
            float v = sv[w2 * MT + tid]; int i = si[w2 * MT + tid];
            if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
        }
        out.part_val[(size_t)blockIdx.x * MAX_ROWS + tid] = bv;
        out.part_idx[(size_t)blockIdx.x * MAX_ROWS + tid] = bi;
    }
    __threadfence();
    __syncthreads();
    __shared__ unsigned s_last;
    if (tid == 0) s_last = (atomicAdd(out.counter, 1u) == gridDim.x - 1) ? 1u : 0u;
    __syncthreads();
    if (s_last) {
        __threadfence();
        if (tid < M) {
            float bv = -INFINITY; int bi = 0x7FFFFFFF;
            for (unsigned g = 0; g < gridDim.x; ++g) {
                float v = __builtin_nontemporal_load(out.part_val + (size_t)g * MAX_ROWS + tid);
                int i = __builtin_nontemporal_load(out.part_idx + (size_t)g * MAX_ROWS + tid);
                if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
            }
            if (out.dst == ROWS_DRAFT) st->d[out.off] = bi;
            else st->amax[tid] = bi;
        }
        if (tid == 0) *out.counter = 0u;
    }
}

// ---- a3: causal attention of M rows over the contiguous cache, split along positions --------------------
// grid (n_splits_max, Hkv).  A workgroup handles one split of ATT_SL positions of one KV head for all rows
// and all query heads of the group; K/V tiles are staged in LDS once.  Partials (max, sum, o) go to the
// workspace; the last workgroup of a KV head to finish merges the splits in ascending order.
struct AttnArgs {
    const float* q;    // [M][H*hd]
    float* att;        // [M][H*hd]
    float* part_o;     // [n_splits][MAX_ROWS][H][hd]
    float* part_ml;    // [n_splits][MAX_ROWS][H][2]
    unsigned* counters;  // [Hkv], left at 0
    LayerDims L;
    Rows rows;
    const DevState* st;
};

template <typename WT>
__global__ __launch_bounds__(256) void k_attn(const WT* __restrict__ kc, const WT* __restrict__ vc, AttnArgs a) {
    extern __shared__ float lds[];
    const int hd = a.L.hd, H = a.L.H, Hkv = a.L.Hkv, grp = H / Hkv, M = a.rows.M;
    const int split = blockIdx.x, g = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pos0 = row_pos(a.rows, a.st, 0);      // position of row 0; row m sits at pos0 + m
    const int Ltot = pos0 + M;                      // positions visible to the last row
    const int n_active = (Ltot + ATT_SL - 1) / ATT_SL;
    if (split >= n_active) return;
    const int start = split * ATT_SL, npos = min(ATT_SL, Ltot - start);
    constexpr int PADB = 16;                        // bytes of padding per staged row (bank spread)
    const int rstride = hd + PADB / (int)sizeof(WT);   // elements
    WT* ks = reinterpret_cast<WT*>(lds);
    WT* vs = ks + ATT_SL * rstride;
    float* qs = reinterpret_cast<float*>(vs + ATT_SL * rstride);   // [ATT_QC][hd]
    float* sc = qs + ATT_QC * hd;                                  // [ATT_QC][ATT_SL]
    const float scale = 1.0f / sqrtf((float)hd);

    // stage K and V tiles (16-byte pieces; rows beyond npos zero-filled)
    constexpr int VEC = ST<WT>::VEC;
    const WT* kg = kc + ((size_t)g * a.L.max_seq + start) * hd;
    const WT* vg = vc + ((size_t)g * a.L.max_seq + start) * hd;
    const int per_row = hd / VEC;
    for (int idx = tid; idx < ATT_SL * per_row; idx += blockDim.x) {
        int j = idx / per_row, c = (idx - j * per_row) * VEC;
        uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
        if (j < npos) {
            kv = *reinterpret_cast<const uint4*>(kg + (size_t)j * hd + c);
            vv = *reinterpret_cast<const uint4*>(vg + (size_t)j * hd + c);
        }
        *reinterpret_cast<uint4*>(ks + j * rstride + c) = kv;
        *reinterpret_cast<uint4*>(vs + j * rstride + c) = vv;
    }
    const int nq = M * grp;   // query vectors: qi = m * grp + gi
    for (int q0 = 0; q0 < nq; q0 += ATT_QC) {
        const int nqc = min(ATT_QC, nq - q0);
        __syncthreads();
        for (int idx = tid; idx < nqc * hd; idx += blockDim.x) {
            int qi = q0 + idx / hd, dim = idx % hd, m = qi / grp, gi = qi - m * grp;
            qs[idx] = a.q[(size_t)m * H * hd + (size_t)(g * grp + gi) * hd + dim] * scale;
        }
        __syncthreads();
        // scores: a thread owns one position and a subset of the queries
        {
            const int j = tid % ATT_SL, qsub = tid / ATT_SL, nsub = blockDim.x / ATT_SL;
            for (int ql = qsub; ql < nqc; ql += nsub) {
                const int m = (q0 + ql) / grp;
                float s = -INFINITY;
                if (j < npos && start + j <= pos0 + m) {
                    s = 0.f;
                    const WT* kr = ks + j * rstride;
                    const float* qv = qs + ql * hd;
                    for (int c = 0; c < hd; c += VEC) {
                        float wf[VEC];
                        ST<WT>::unpack(*reinterpret_cast<const uint4*>(kr + c), wf);
#pragma unroll
                        for (int v = 0; v < VEC; ++v) s = fmaf(wf[v], qv[c + v], s);
                    }
                }
                sc[ql * ATT_SL + j] = s;
            }
        }
        __syncthreads();
        // soft-max statistics per query (one wave per query), probabilities written back in place
        for (int ql = wave; ql < nqc; ql += (blockDim.x >> 6)) {
            float s0 = sc[ql * ATT_SL + lane], s1 = sc[ql * ATT_SL + 64 + lane];
            float mx = wave_max(fmaxf(s0, s1));
            float p0 = 0.f, p1 = 0.f;
            if (mx > -INFINITY) { p0 = __expf(s0 - mx); p1 = __expf(s1 - mx); }
            sc[ql * ATT_SL + lane] = p0; sc[ql * ATT_SL + 64 + lane] = p1;
            // sum in position order inside each lane pair, then the fixed butterfly
            float l = wave_sum(p0 + p1);
            if (lane == 0) {
                const int qi = q0 + ql, m = qi / grp, hq = g * grp + (qi - m * grp);
                float* ml = a.part_ml + (((size_t)split * MAX_ROWS + m) * H + hq) * 2;
                ml[0] = mx; ml[1] = l;
            }
        }
        __syncthreads();
        // o[dim] = sum_j p[j] * V[j][dim]; a thread owns one dim and a subset of the queries
        {
            const int dim = tid % hd, qsub = tid / hd, nsub = blockDim.x / hd;
            for (int ql = qsub; ql < nqc; ql += nsub) {
                float o = 0.f;
                const float* p = sc + ql * ATT_SL;
                for (int j = 0; j < npos; ++j) o = fmaf(p[j], ST<WT>::ld(vs + j * rstride + dim), o);
                const int qi = q0 + ql, m = qi / grp, hq = g * grp + (qi - m * grp);
                a.part_o[(((size_t)split * MAX_ROWS + m) * H + hq) * hd + dim] = o;
            }
        }
    }
    // last workgroup of this KV head merges the splits
    __threadfence();
    __syncthreads();
    __shared__ unsigned s_last;
    if (tid == 0) s_last = (atomicAdd(a.counters + g, 1u) == (unsigned)(n_active - 1)) ? 1u : 0u;
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    for (int idx = tid; idx < nq * hd; idx += blockDim.x) {
        const int qi = idx / hd, dim = idx - qi * hd, m = qi / grp, hq = g * grp + (qi - m * grp);
        float gmax = -INFINITY;
        for (int s = 0; s < n_active; ++s)
            gmax = fmaxf(gmax, __builtin_nontemporal_load(a.part_ml + (((size_t)s * MAX_ROWS + m) * H + hq) * 2));
        float num = 0.f, den = 0.f;
        for (int s = 0; s < n_active; ++s) {
            const float* ml = a.part_ml + (((size_t)s * MAX_ROWS + m) * H + hq) * 2;
            const float ms = __builtin_nontemporal_load(ml), ls = __builtin_nontemporal_load(ml + 1);
            const float w = (ms > -INFINITY) ? __expf(ms - gmax) : 0.f;
            const float o = __builtin_nontemporal_load(a.part_o + (((size_t)s * MAX_ROWS + m) * H + hq) * hd + dim);
            num = fmaf(w, o, num);
            den = fmaf(w, ls, den);
        }
        a.att[(size_t)m * H * hd + (size_t)hq * hd + dim] = num / den;
    }
    if (tid == 0) a.counters[g] = 0u;
}

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
