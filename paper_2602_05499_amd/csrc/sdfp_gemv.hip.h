// Weight-streaming skinny GEMM of the forward pass and its fused prologues / epilogues:
//   a2  RMSNorm -> QKV projection -> RoPE -> KV append
//   a4  O projection + residual           a6  down projection + residual
//   a5  RMSNorm -> gate/up projection -> SiLU * mul
//   a7  final RMSNorm -> output projection -> arg-max partials
#pragma once
#include "sdfp_common.hip.h"

namespace sdfp {

// Y[m][n] = sum_k W[n][k] * X[m][k] for M <= MT rows.
//
// Work decomposition.  Output rows are grouped in UNITS of two rows (the two rows a fused epilogue needs
// together: a rotary pair, a gate/up pair, or two consecutive rows).  Each workgroup owns a contiguous
// range of units and walks it in batches of 8 units, one unit per wave.  A wave streams its two weight
// rows over the whole K range: lanes split K in 16-byte pieces (64 lanes x 16 B = one CHUNK, a fully
// coalesced 1 KB read per row), D chunks are kept in flight in a register ring that runs ahead across unit
// boundaries -- and, in the single-kernel forward, across phase boundaries -- so the HBM queue never drains.
// X is staged in LDS (once per phase when a whole row fits the budget, else tile by tile), laid out so that
// every lane's 16-byte LDS reads are conflict-free.  Per-lane partial sums are float32 FMAs in
// ascending-chunk order; the cross-lane sum is a fixed DPP tree.  Nothing in this order depends on M.
// Epilogues issue no global loads (a load would make the wave wait for its whole prefetch ring): what they
// need (rotary table rows, residual values) is staged in LDS at the start of the phase.
template <typename WT> struct Chunk {
    static constexpr int VEC = ST<WT>::VEC;
    static constexpr int ELEMS = 64 * VEC;   // K elements per chunk (bf16 512, f32 256)
};

constexpr int GEMV_RED_FLOATS = NWAVE * MAX_ROWS + MAX_ROWS + 7;   // norm reduction scratch
constexpr int GEMV_EX_FLOATS = 2560;                               // per-phase epilogue staging
constexpr size_t GEMV_LDS_BYTES = XS_BUDGET_BYTES + (GEMV_RED_FLOATS + GEMV_EX_FLOATS) * 4;

struct GemvGeom {
    int C;        // chunks per weight row
    int CT;       // chunks per LDS tile
    int T;        // tiles
    int u0, u1;   // this workgroup's unit range
    int nb;       // batches of NWAVE units
    int total;    // steps per wave = nb * C
};

template <typename WT, int MT>
__device__ __forceinline__ GemvGeom gemv_geom(int n_units, int Kd, int wg, int n_wg) {
    GemvGeom g;
    g.C = (Kd + Chunk<WT>::ELEMS - 1) / Chunk<WT>::ELEMS;
    const int fit = XS_BUDGET_BYTES / (MT * Chunk<WT>::ELEMS * 4);
    g.CT = g.C < fit ? g.C : fit;
    g.T = (g.C + g.CT - 1) / g.CT;
    g.u0 = (int)(((long long)n_units * wg) / n_wg);
    g.u1 = (int)(((long long)n_units * (wg + 1)) / n_wg);
    g.nb = (g.u1 - g.u0 + NWAVE - 1) / NWAVE;
    g.total = g.nb * g.C;
    return g;
}

// index of element k (relative to its tile) inside a staged row: [chunk][piece][lane][4 floats]
template <typename WT>
__device__ __forceinline__ int xs_index(int k) {
    if (Chunk<WT>::VEC == 8) {
        const int chunk = k >> 9, lane = (k >> 3) & 63, half = (k >> 2) & 1, j = k & 3;
        return ((chunk * 2 + half) * 64 + lane) * 4 + j;
    }
    return k;   // VEC == 4: one 16-byte piece per lane per chunk, natural order
}

template <int D> struct Ring { u32x4 r[D][2]; };

// 1 KB chunks kept in flight per weight row and wave (register ring depth), by row count of the forward:
// the fewer activation rows, the more registers are free to run ahead of the dependency chain of a phase
// boundary (store acknowledgement, barrier, activation staging).
__host__ __device__ constexpr int ring_depth(int MT) { return MT <= 2 ? 16 : (MT <= 6 ? 8 : 4); }

// Op concept:
//   int  n_units() const;  int Kd() const;  int rows() const;
//   void wrows(int unit, const WT* (&r)[2]) const;                 weight rows of a unit
//   void pre(float* ex, const GemvGeom& g) const;                  all threads: stage epilogue inputs in LDS
//   void done(int unit, float (&acc)[2][MT], const float* ex, const GemvGeom& g);   lane 63 only
template <typename WT, int MT, int D, class Op>
struct GemvPhase {
    static constexpr int VEC = Chunk<WT>::VEC, CE = Chunk<WT>::ELEMS;
    GemvGeom g;
    int Kd, M, lane, wave;

    __device__ __forceinline__ void setup(const Op& op, int wg, int n_wg) {
        g = gemv_geom<WT, MT>(op.n_units(), op.Kd(), wg, n_wg);
        Kd = op.Kd(); M = op.rows();
        lane = threadIdx.x & 63; wave = threadIdx.x >> 6;
    }

    __device__ __forceinline__ void load_step(const Op& op, int t, u32x4 (&dst)[2]) const {
        dst[0] = u32x4{0, 0, 0, 0};
        dst[1] = u32x4{0, 0, 0, 0};
        if (t < g.total) {
            const int b = t / g.C, c = t - b * g.C;
            const int unit = g.u0 + b * NWAVE + wave;
            const int k = (c * 64 + lane) * VEC;
            if (unit < g.u1 && k < Kd) {
                const WT* r[2];
                op.wrows(unit, r);
                dst[0] = ld_stream(r[0] + k);
                dst[1] = ld_stream(r[1] + k);
            }
        }
    }

    // issue the first D steps' weight loads (they depend on nothing a previous phase computes)
    __device__ __forceinline__ void prefetch(const Op& op, Ring<D>& ring) const {
#pragma unroll
        for (int d = 0; d < D; ++d) load_step(op, d, ring.r[d]);
    }

    // stage tile `tile` of X (optionally multiplied by the norm gain) into LDS; when want_ss, adds the
    // squares of the raw values this thread touched to ss[row]
    __device__ __forceinline__ void stage(const float* __restrict__ xsrc, const float* __restrict__ gain, float* xs,
                                          int tile, float (&ss)[MT], bool want_ss) const {
        const int k_lo = tile * g.CT * CE, k_hi = min(Kd, k_lo + g.CT * CE), klen = k_hi - k_lo;
        const int row_floats = g.CT * CE;
        const int padded = ((klen + CE - 1) / CE) * CE;
        for (int idx = threadIdx.x * 4; idx < MT * padded; idx += WG_THREADS * 4) {
            const int m = idx / padded, kk = idx - m * padded;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (m < M && kk < klen) {
                v = ld_coh4(xsrc + (size_t)m * Kd + k_lo + kk);
                if (want_ss) {
                    const float s = v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
#pragma unroll
                    for (int mm = 0; mm < MT; ++mm)
                        if (mm == m) ss[mm] += s;
                }
                if (gain != nullptr) v = v * *reinterpret_cast<const f32x4*>(gain + k_lo + kk);
            }
            *reinterpret_cast<f32x4*>(__builtin_assume_aligned(xs + m * row_floats + xs_index<WT>(kk), 16)) = v;
        }
    }

    // lds: [xs: XS_BUDGET_BYTES][red: GEMV_RED_FLOATS][ex: GEMV_EX_FLOATS].  The ring must hold steps 0..D-1.
    __device__ __forceinline__ void run(Op& op, Ring<D>& ring, const float* __restrict__ xsrc,
                                        const float* __restrict__ gain, float eps, float* lds) {
        if (g.total == 0) return;   // uniform over the workgroup
        float* xs = lds;
        float* red = lds + XS_BUDGET_BYTES / 4;
        float* ex = red + GEMV_RED_FLOATS;
        const int row_floats = g.CT * CE;
        float* rs = red + NWAVE * MT;   // [MT] reciprocal RMS (applied to the accumulators in the epilogue)
        const bool norm = gain != nullptr;
        float ss[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) ss[m] = 0.f;

        op.pre(ex, g);
        if (norm && g.T > 1) {   // the row does not fit one tile: separate pass for the sum of squares
            for (int idx = threadIdx.x * 4; idx < M * Kd; idx += WG_THREADS * 4) {
                const int m = idx / Kd;
                const f32x4 v = ld_coh4(xsrc + idx);
                const float s = v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
#pragma unroll
                for (int mm = 0; mm < MT; ++mm)
                    if (mm == m) ss[mm] += s;
            }
        }
        float acc[2][MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) { acc[0][m] = 0.f; acc[1][m] = 0.f; }

        int c = 0, b = 0;
        bool first = true;
        for (int t0 = 0; t0 < g.total; t0 += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const int t = t0 + d;
                if (t < g.total) {
                    const int ct = c % g.CT;
                    if (ct == 0 && (g.T > 1 || first)) {   // (re)stage the tile this chunk belongs to
                        if (!first) __syncthreads();
                        stage(xsrc, gain, xs, c / g.CT, ss, norm && g.T == 1 && first);
                        if (first) {
                            if (norm) {
#pragma unroll
                                for (int m = 0; m < MT; ++m) {
                                    const float s = wave_sum_last(ss[m]);
                                    if (lane == 63) red[wave * MT + m] = s;
                                }
                            }
                            __syncthreads();
                            if (norm && threadIdx.x < MT) {
                                float s = 0.f;
                                for (int w = 0; w < NWAVE; ++w) s += red[w * MT + threadIdx.x];
                                rs[threadIdx.x] = 1.0f / sqrtf(s / (float)Kd + eps);
                            }
                            first = false;
                        }
                        __syncthreads();
                    }
                    const u32x4 cur0 = ring.r[d][0], cur1 = ring.r[d][1];
                    load_step(op, t + D, ring.r[d]);
                    float xv[MT][VEC];
#pragma unroll
                    for (int m = 0; m < MT; ++m)
#pragma unroll
                        for (int p = 0; p < VEC / 4; ++p) {
                            const f32x4 a = *reinterpret_cast<const f32x4*>(__builtin_assume_aligned(
                                xs + m * row_floats + ((ct * (VEC / 4) + p) * 64 + lane) * 4, 16));
                            xv[m][p * 4 + 0] = a.x; xv[m][p * 4 + 1] = a.y; xv[m][p * 4 + 2] = a.z; xv[m][p * 4 + 3] = a.w;
                        }
                    float wf[VEC];
                    ST<WT>::unpack(cur0, wf);
#pragma unroll
                    for (int m = 0; m < MT; ++m)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) acc[0][m] = fmaf(wf[v], xv[m][v], acc[0][m]);
                    ST<WT>::unpack(cur1, wf);
#pragma unroll
                    for (int m = 0; m < MT; ++m)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) acc[1][m] = fmaf(wf[v], xv[m][v], acc[1][m]);
                    if (++c == g.C) {   // unit finished: reduce over lanes, epilogue in lane 63
                        c = 0;
                        const int unit = g.u0 + b * NWAVE + wave;
#pragma unroll
                        for (int m = 0; m < MT; ++m) {
                            acc[0][m] = wave_sum_last(acc[0][m]);
                            acc[1][m] = wave_sum_last(acc[1][m]);
                        }
                        if (lane == 63 && unit < g.u1) {
                            if (norm) {
#pragma unroll
                                for (int m = 0; m < MT; ++m) { acc[0][m] *= rs[m]; acc[1][m] *= rs[m]; }
                            }
                            op.done(unit, acc, ex, g);
                        }
#pragma unroll
                        for (int m = 0; m < MT; ++m) { acc[0][m] = 0.f; acc[1][m] = 0.f; }
                        ++b;
                    }
                }
            }
        }
    }
};

// ---- a2: RMSNorm -> QKV projection -> RoPE -> KV append ------------------------------------------------
// Unit = the rotary pair (i, i + hd/2) of one head of the concatenated [Wq; Wk; Wv] row space.
template <typename WT, int MT>
struct QkvOp {
    const WT *wq, *wk, *wv;
    WT *kc, *vc;               // this layer's K and V cache planes [Hkv][max_seq][hd]
    float* q;                  // [M][H*hd]
    const float *cosT, *sinT;  // [max_seq][hd/2]
    LayerDims L;
    int M, pos0;               // rows and the position of row 0 (row m sits at pos0 + m)
    __device__ __forceinline__ int n_units() const { return (L.H + 2 * L.Hkv) * (L.hd >> 1); }
    __device__ __forceinline__ int Kd() const { return L.d; }
    __device__ __forceinline__ int rows() const { return M; }
    __device__ __forceinline__ void wrows(int unit, const WT* (&r)[2]) const {
        const int half = L.hd >> 1, hs = unit / half, i = unit - hs * half;
        const WT* base;
        if (hs < L.H) base = wq + (size_t)hs * L.hd * L.d;
        else if (hs < L.H + L.Hkv) base = wk + (size_t)(hs - L.H) * L.hd * L.d;
        else base = wv + (size_t)(hs - L.H - L.Hkv) * L.hd * L.d;
        r[0] = base + (size_t)i * L.d;
        r[1] = base + (size_t)(i + half) * L.d;
    }
    // rotary rows of the M positions: ex[(m * half + i) * 2 + {0: cos, 1: sin}]
    __device__ __forceinline__ void pre(float* ex, const GemvGeom&) const {
        const int half = L.hd >> 1;
        for (int idx = threadIdx.x; idx < M * half; idx += WG_THREADS) {
            const int m = idx / half, i = idx - m * half;
            ex[idx * 2] = cosT[(size_t)(pos0 + m) * half + i];
            ex[idx * 2 + 1] = sinT[(size_t)(pos0 + m) * half + i];
        }
    }
    __device__ __forceinline__ void done(int unit, float (&acc)[2][MT], const float* ex, const GemvGeom&) const {
        const int half = L.hd >> 1, hs = unit / half, i = unit - hs * half;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            if (m < M) {
                float a = acc[0][m], b = acc[1][m];
                if (hs < L.H + L.Hkv) {   // rotary: (a, b) -> (a cos - b sin, b cos + a sin)
                    const float c = ex[(m * half + i) * 2], s = ex[(m * half + i) * 2 + 1];
                    const float ra = a * c - b * s, rb = b * c + a * s;
                    a = ra; b = rb;
                }
                if (hs < L.H) {
                    float* o = q + (size_t)m * L.H * L.hd + (size_t)hs * L.hd;
                    st_coh(o + i, a); st_coh(o + i + half, b);
                } else {
                    const bool isk = hs < L.H + L.Hkv;
                    const int kvh = isk ? hs - L.H : hs - L.H - L.Hkv;
                    WT* o = (isk ? kc : vc) + ((size_t)kvh * L.max_seq + pos0 + m) * L.hd;
                    ST<WT>::stc(o + i, a); ST<WT>::stc(o + i + half, b);
                }
            }
        }
    }
};

// ---- a4 / a6: projection + residual add ----------------------------------------------------------------
template <typename WT, int MT>
struct ResidOp {
    const WT* w;   // [N][Kd]
    float* h;      // [M][N] residual stream, updated in place
    int N, K, M;
    __device__ __forceinline__ int n_units() const { return (N + 1) >> 1; }
    __device__ __forceinline__ int Kd() const { return K; }
    __device__ __forceinline__ int rows() const { return M; }
    __device__ __forceinline__ void wrows(int unit, const WT* (&r)[2]) const {
        r[0] = w + (size_t)(unit * 2) * K;
        r[1] = w + (size_t)min(unit * 2 + 1, N - 1) * K;
    }
    __device__ __forceinline__ bool staged(const GemvGeom& g) const { return M * 2 * (g.u1 - g.u0) <= GEMV_EX_FLOATS; }
    // residual values of this workgroup's output rows: ex[m * span + (row - 2 u0)]
    __device__ __forceinline__ void pre(float* ex, const GemvGeom& g) const {
        if (!staged(g)) return;
        const int span = 2 * (g.u1 - g.u0), r0 = 2 * g.u0;
        for (int idx = threadIdx.x; idx < M * span; idx += WG_THREADS) {
            const int m = idx / span, j = idx - m * span;
            ex[idx] = (r0 + j < N) ? ld_coh(h + (size_t)m * N + r0 + j) : 0.f;
        }
    }
    __device__ __forceinline__ void done(int unit, float (&acc)[2][MT], const float* ex, const GemvGeom& g) const {
        const bool st = staged(g);
        const int span = 2 * (g.u1 - g.u0), j = 2 * (unit - g.u0);
#pragma unroll
        for (int m = 0; m < MT; ++m)
            if (m < M) {
                float* o = h + (size_t)m * N + unit * 2;
                st_coh(o, (st ? ex[m * span + j] : ld_coh(o)) + acc[0][m]);
                if (unit * 2 + 1 < N) st_coh(o + 1, (st ? ex[m * span + j + 1] : ld_coh(o + 1)) + acc[1][m]);
            }
    }
};

// ---- a5: RMSNorm -> gate/up projection -> SiLU * mul ---------------------------------------------------
// Unit j = (gate row j, up row j).
template <typename WT, int MT>
struct GateUpOp {
    const WT *wg, *wu;   // [F][d]
    float* a;            // [M][F]
    int F, d, M;
    __device__ __forceinline__ int n_units() const { return F; }
    __device__ __forceinline__ int Kd() const { return d; }
    __device__ __forceinline__ int rows() const { return M; }
    __device__ __forceinline__ void wrows(int unit, const WT* (&r)[2]) const {
        r[0] = wg + (size_t)unit * d;
        r[1] = wu + (size_t)unit * d;
    }
    __device__ __forceinline__ void pre(float*, const GemvGeom&) const {}
    __device__ __forceinline__ void done(int unit, float (&acc)[2][MT], const float*, const GemvGeom&) const {
#pragma unroll
        for (int m = 0; m < MT; ++m)
            if (m < M) {
                const float g = acc[0][m], u = acc[1][m];
                st_coh(a + (size_t)m * F + unit, (g / (1.0f + __expf(-g))) * u);
            }
    }
};

// ---- a7: final RMSNorm -> output projection -> fused arg-max -------------------------------------------
// Lane 63 of every wave keeps the running (max, lowest index) of the rows it produced; workgroups publish
// partials and a final pass reduces them (lowest index wins ties) and writes the token(s).
struct HeadOut {
    float* logits;        // [M][V] or nullptr
    float* part_val;      // [n_wg][MAX_ROWS]
    int* part_idx;        // [n_wg][MAX_ROWS]
    unsigned* counter;    // arrival counter of the separate-kernel path (left at 0)
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
    __device__ __forceinline__ int n_units() const { return (V + 1) >> 1; }
    __device__ __forceinline__ int Kd() const { return d; }
    __device__ __forceinline__ int rows() const { return M; }
    __device__ __forceinline__ void init(const WT* w_, int V_, int d_, int M_, float* logits_) {
        w = w_; V = V_; d = d_; M = M_; logits = logits_;
#pragma unroll
        for (int m = 0; m < MT; ++m) { best_v[m] = -INFINITY; best_i[m] = 0x7FFFFFFF; }
    }
    __device__ __forceinline__ void wrows(int unit, const WT* (&r)[2]) const {
        r[0] = w + (size_t)(unit * 2) * d;
        r[1] = w + (size_t)min(unit * 2 + 1, V - 1) * d;
    }
    __device__ __forceinline__ void pre(float*, const GemvGeom&) const {}
    __device__ __forceinline__ void done(int unit, float (&acc)[2][MT], const float*, const GemvGeom&) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = unit * 2 + j;
            if (n < V) {
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    const float v = acc[j][m];
                    if (v > best_v[m] || (v == best_v[m] && n < best_i[m])) { best_v[m] = v; best_i[m] = n; }
                    if (logits != nullptr && m < M) logits[(size_t)m * V + n] = v;
                }
            }
        }
    }
};

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

// workgroup reduce of the per-wave bests (held by lane 63 of each wave) -> this workgroup's partial
template <typename WT, int MT>
__device__ __forceinline__ void head_publish(const HeadOp<WT, MT>& op, const HeadOut& out, float* lds, int wg) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __syncthreads();
    float* sv = lds;                                              // [NWAVE][MT]
    int* si = reinterpret_cast<int*>(lds + NWAVE * MAX_ROWS);     // [NWAVE][MT]
    if (lane == 63)
#pragma unroll
        for (int m = 0; m < MT; ++m) { sv[wave * MT + m] = op.best_v[m]; si[wave * MT + m] = op.best_i[m]; }
    __syncthreads();
    if (tid < op.M) {
        float bv = -INFINITY; int bi = 0x7FFFFFFF;
        for (int w2 = 0; w2 < NWAVE; ++w2) {
            const float v = sv[w2 * MT + tid]; const int i = si[w2 * MT + tid];
            if (better(v, i, bv, bi)) { bv = v; bi = i; }
        }
        st_coh(out.part_val + (size_t)wg * MAX_ROWS + tid, bv);
        st_coh(out.part_idx + (size_t)wg * MAX_ROWS + tid, bi);
    }
    stores_done();
}

// final reduce over the n_wg partials by one workgroup: wave m handles row m
__device__ __forceinline__ void head_final(const HeadOut& out, int M, int n_wg, DevState* st) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int m = wave; m < M; m += NWAVE) {
        float bv = -INFINITY; int bi = 0x7FFFFFFF;
        for (int g = lane; g < n_wg; g += 64) {
            const float v = ld_coh(out.part_val + (size_t)g * MAX_ROWS + m);
            const int i = ld_coh(out.part_idx + (size_t)g * MAX_ROWS + m);
            if (better(v, i, bv, bi)) { bv = v; bi = i; }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float v = __shfl_xor(bv, off); const int i = __shfl_xor(bi, off);
            if (better(v, i, bv, bi)) { bv = v; bi = i; }
        }
        if (lane == 0) {
            if (out.dst == ROWS_DRAFT) st->d[out.off] = bi;
            else st->amax[m] = bi;
        }
    }
}

// ---- one kernel per phase (fallback path and prompt processing) -----------------------------------------
template <typename WT, int MT, int D>
__global__ __launch_bounds__(WG_THREADS, 1) void k_qkv(QkvOp<WT, MT> op, Rows rows, const DevState* st,
                                                       const float* __restrict__ h, const float* __restrict__ gain,
                                                       float eps) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    op.M = rows.M; op.pos0 = row_pos(rows, st, 0);
    GemvPhase<WT, MT, D, QkvOp<WT, MT>> ph;
    Ring<D> ring;
    ph.setup(op, blockIdx.x, gridDim.x);
    ph.prefetch(op, ring);
    ph.run(op, ring, h, gain, eps, lds);
}

template <typename WT, int MT, int D>
__global__ __launch_bounds__(WG_THREADS, 1) void k_resid(ResidOp<WT, MT> op, const float* __restrict__ x) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    GemvPhase<WT, MT, D, ResidOp<WT, MT>> ph;
    Ring<D> ring;
    ph.setup(op, blockIdx.x, gridDim.x);
    ph.prefetch(op, ring);
    ph.run(op, ring, x, nullptr, 0.f, lds);
}

template <typename WT, int MT, int D>
__global__ __launch_bounds__(WG_THREADS, 1) void k_gateup(GateUpOp<WT, MT> op, const float* __restrict__ h,
                                                          const float* __restrict__ gain, float eps) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    GemvPhase<WT, MT, D, GateUpOp<WT, MT>> ph;
    Ring<D> ring;
    ph.setup(op, blockIdx.x, gridDim.x);
    ph.prefetch(op, ring);
    ph.run(op, ring, h, gain, eps, lds);
}

template <typename WT, int MT, int D>
__global__ __launch_bounds__(WG_THREADS, 1) void k_head(const WT* __restrict__ w, const float* __restrict__ h,
                                                        const float* __restrict__ gain, float eps, int V, int d,
                                                        int M, HeadOut out, DevState* st) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    HeadOp<WT, MT> op;
    op.init(w, V, d, M, out.logits);
    GemvPhase<WT, MT, D, HeadOp<WT, MT>> ph;
    Ring<D> ring;
    ph.setup(op, blockIdx.x, gridDim.x);
    ph.prefetch(op, ring);
    ph.run(op, ring, h, gain, eps, lds);
    head_publish(op, out, lds, blockIdx.x);
    __syncthreads();   // every wave's coherent stores are acknowledged before the arrival is counted
    __shared__ unsigned s_last;
    if (threadIdx.x == 0) s_last = (atomicAdd(out.counter, 1u) == gridDim.x - 1) ? 1u : 0u;
    __syncthreads();
    if (!s_last) return;
    head_final(out, M, gridDim.x, st);
    if (threadIdx.x == 0) st_coh(out.counter, 0u);
}

}  // namespace sdfp
