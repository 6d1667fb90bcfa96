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
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int MAX_K = 8;
constexpr int MAX_ROWS = MAX_K + 1;
constexpr int WG_THREADS = 512;  // every forward-pass kernel runs 8 waves per workgroup, one workgroup per CU
constexpr int NWAVE = WG_THREADS / 64;
constexpr int ATT_SL = 128;      // attention split length in positions (fixed absolute boundaries)
constexpr int ATT_QC = 16;       // query vectors processed per pass inside an attention workgroup
constexpr int XS_BUDGET_BYTES = 144 * 1024;   // LDS given to the staged activations of a projection phase

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
    static __device__ __forceinline__ void unpack(const u32x4& r, float (&w)[4]) {
        w[0] = __uint_as_float(r.x); w[1] = __uint_as_float(r.y);
        w[2] = __uint_as_float(r.z); w[3] = __uint_as_float(r.w);
    }
};
template <> struct ST<bf16_t> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
    static __device__ __forceinline__ void unpack(const u32x4& r, float (&w)[8]) {
        w[0] = __uint_as_float(r.x << 16); w[1] = __uint_as_float(r.x & 0xFFFF0000u);
        w[2] = __uint_as_float(r.y << 16); w[3] = __uint_as_float(r.y & 0xFFFF0000u);
        w[4] = __uint_as_float(r.z << 16); w[5] = __uint_as_float(r.z & 0xFFFF0000u);
        w[6] = __uint_as_float(r.w << 16); w[7] = __uint_as_float(r.w & 0xFFFF0000u);
    }
};

// streaming (read-once) 16-byte weight load
__device__ __forceinline__ u32x4 ld_stream(const void* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

// ---- wave64 reductions on the DPP network (no LDS traffic).  The total lands in the LAST lane of each
// group of G consecutive lanes (G a power of two, 2..64); the summation tree is fixed. -------------------
template <int CTRL, int ROWMASK>
__device__ __forceinline__ float dpp_add(float v) {
    return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWMASK,
                                                                      0xf, false));
}
template <int G>
__device__ __forceinline__ float group_sum_dpp(float v) {
    if (G >= 2) v = dpp_add<0x111, 0xf>(v);    // row_shr:1
    if (G >= 4) v = dpp_add<0x112, 0xf>(v);    // row_shr:2
    if (G >= 8) v = dpp_add<0x114, 0xf>(v);    // row_shr:4
    if (G >= 16) v = dpp_add<0x118, 0xf>(v);   // row_shr:8
    if (G >= 32) v = dpp_add<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    if (G >= 64) v = dpp_add<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ __forceinline__ float wave_sum_last(float v) { return group_sum_dpp<64>(v); }   // valid in lane 63

__device__ __forceinline__ float wave_sum(float v) {   // butterfly: total in every lane
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
// Y[m][n] = sum_k W[n][k] * X[m][k] for M <= MT rows.
//
// Work decomposition.  Output rows are grouped in UNITS of two rows (the two rows a fused epilogue needs
// together: a rotary pair, a gate/up pair, or two consecutive rows).  Each workgroup owns a contiguous
// range of units and walks it in batches of 8 units, one unit per wave.  A wave streams its two weight
// rows over the whole K range: lanes split K in 16-byte pieces (64 lanes x 16 B = one CHUNK, a fully
// coalesced 1 KB read per row), D chunks are kept in flight in a register ring that runs ahead across unit
// boundaries, so the HBM queue never drains inside a phase.  X is staged in LDS (once per phase when a whole
// row fits the budget, else tile by tile), laid out so that every lane's 16-byte LDS reads are
// conflict-free.  Per-lane partial sums are float32 FMAs in ascending-chunk order; the cross-lane sum is a
// fixed DPP tree.  Nothing in this order depends on M.
template <typename WT> struct Chunk {
    static constexpr int VEC = ST<WT>::VEC;
    static constexpr int ELEMS = 64 * VEC;   // K elements per chunk (bf16 512, f32 256)
};

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

// Op concept:
//   void wrows(int unit, const WT* (&r)[2]) const;          weight rows of a unit
//   void done(int unit, float (&acc)[2][MT]);               epilogue, executed by lane 63 only
template <typename WT, int MT, int D, class Op>
struct GemvPhase {
    static constexpr int VEC = Chunk<WT>::VEC, CE = Chunk<WT>::ELEMS;
    GemvGeom g;
    int Kd, M, lane, wave;
    u32x4 ring[D][2];

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

    __device__ __forceinline__ void setup(int n_units, int Kd_, int M_, int wg, int n_wg) {
        g = gemv_geom<WT, MT>(n_units, Kd_, wg, n_wg);
        Kd = Kd_; M = M_;
        lane = threadIdx.x & 63; wave = threadIdx.x >> 6;
    }

    // issue the first D steps' weight loads (they depend on nothing a previous phase computes)
    __device__ __forceinline__ void prefetch(const Op& op) {
#pragma unroll
        for (int d = 0; d < D; ++d) load_step(op, d, ring[d]);
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
                v = *reinterpret_cast<const f32x4*>(xsrc + (size_t)m * Kd + k_lo + kk);
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

    // xs: LDS for the staged rows (MT * CT * CE floats); red: LDS scratch (NWAVE * MT + MT floats)
    __device__ __forceinline__ void run(Op& op, const float* __restrict__ xsrc, const float* __restrict__ gain,
                                        float eps, float* xs, float* red) {
        if (g.total == 0) return;   // uniform over the workgroup
        const int row_floats = g.CT * CE;
        float* rs = red + NWAVE * MT;   // [MT] reciprocal RMS (applied to the accumulators in the epilogue)
        const bool norm = gain != nullptr;
        float ss[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) ss[m] = 0.f;

        if (norm && g.T > 1) {   // the row does not fit one tile: separate pass for the sum of squares
            for (int idx = threadIdx.x * 4; idx < M * Kd; idx += WG_THREADS * 4) {
                const int m = idx / Kd;
                const f32x4 v = *reinterpret_cast<const f32x4*>(xsrc + idx);
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
                    const u32x4 cur0 = ring[d][0], cur1 = ring[d][1];
                    load_step(op, t + D, ring[d]);
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
                            op.done(unit, acc);
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

constexpr int GEMV_RED_FLOATS = NWAVE * MAX_ROWS + MAX_ROWS + 7;
constexpr size_t GEMV_LDS_BYTES = XS_BUDGET_BYTES + GEMV_RED_FLOATS * 4;

struct LayerDims {
    int d, H, Hkv, hd, F, V, max_seq;
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
    Rows rows;
    const DevState* st;
    __device__ __forceinline__ void wrows(int unit, const WT* (&r)[2]) const {
        const int half = L.hd >> 1, hs = unit / half, i = unit - hs * half;
        const WT* base;
        if (hs < L.H) base = wq + (size_t)hs * L.hd * L.d;
        else if (hs < L.H + L.Hkv) base = wk + (size_t)(hs - L.H) * L.hd * L.d;
        else base = wv + (size_t)(hs - L.H - L.Hkv) * L.hd * L.d;
        r[0] = base + (size_t)i * L.d;
        r[1] = base + (size_t)(i + half) * L.d;
    }
    __device__ __forceinline__ void done(int unit, float (&acc)[2][MT]) const {
        const int half = L.hd >> 1, hs = unit / half, i = unit - hs * half;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            if (m < rows.M) {
                const int pos = row_pos(rows, st, m);
                float a = acc[0][m], b = acc[1][m];
                if (hs < L.H + L.Hkv) {   // rotary: (a, b) -> (a cos - b sin, b cos + a sin)
                    const float c = cosT[(size_t)pos * half + i], s = sinT[(size_t)pos * half + i];
                    const float ra = a * c - b * s, rb = b * c + a * s;
                    a = ra; b = rb;
                }
                if (hs < L.H) {
                    float* o = q + (size_t)m * L.H * L.hd + (size_t)hs * L.hd;
                    o[i] = a; o[i + half] = b;
                } else {
                    const bool isk = hs < L.H + L.Hkv;
                    const int kvh = isk ? hs - L.H : hs - L.H - L.Hkv;
                    WT* o = (isk ? kc : vc) + ((size_t)kvh * L.max_seq + pos) * L.hd;
                    ST<WT>::st(o + i, a); ST<WT>::st(o + i + half, b);
                }
            }
        }
    }
};

template <typename WT, int MT, int D>
__global__ __launch_bounds__(WG_THREADS, 1) void k_qkv(QkvOp<WT, MT> op, const float* __restrict__ h,
                                                       const float* __restrict__ gain, float eps) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    GemvPhase<WT, MT, D, QkvOp<WT, MT>> ph;
    ph.setup((op.L.H + 2 * op.L.Hkv) * (op.L.hd >> 1), op.L.d, op.rows.M, blockIdx.x, gridDim.x);
    ph.prefetch(op);
    ph.run(op, h, gain, eps, lds, lds + XS_BUDGET_BYTES / 4);
}

// ---- a4 / a6: projection + residual add ----------------------------------------------------------------
template <typename WT, int MT>
struct ResidOp {
    const WT* w;   // [N][Kd]
    float* h;      // [M][N] residual stream, updated in place
    int N, Kd, M;
    __device__ __forceinline__ void wrows(int unit, const WT* (&r)[2]) const {
        r[0] = w + (size_t)(unit * 2) * Kd;
        r[1] = w + (size_t)min(unit * 2 + 1, N - 1) * Kd;
    }
    __device__ __forceinline__ void done(int unit, float (&acc)[2][MT]) const {
#pragma unroll
        for (int m = 0; m < MT; ++m)
            if (m < M) {
                h[(size_t)m * N + unit * 2] += acc[0][m];
                if (unit * 2 + 1 < N) h[(size_t)m * N + unit * 2 + 1] += acc[1][m];
            }
    }
};

template <typename WT, int MT, int D>
__global__ __launch_bounds__(WG_THREADS, 1) void k_resid(ResidOp<WT, MT> op, const float* __restrict__ x) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    GemvPhase<WT, MT, D, ResidOp<WT, MT>> ph;
    ph.setup((op.N + 1) / 2, op.Kd, op.M, blockIdx.x, gridDim.x);
    ph.prefetch(op);
    ph.run(op, x, nullptr, 0.f, lds, lds + XS_BUDGET_BYTES / 4);
}

// ---- a5: RMSNorm -> gate/up projection -> SiLU * mul ---------------------------------------------------
// Unit j = (gate row j, up row j).
template <typename WT, int MT>
struct GateUpOp {
    const WT *wg, *wu;   // [F][d]
    float* a;            // [M][F]
    int F, d, M;
    __device__ __forceinline__ void wrows(int unit, const WT* (&r)[2]) const {
        r[0] = wg + (size_t)unit * d;
        r[1] = wu + (size_t)unit * d;
    }
    __device__ __forceinline__ void done(int unit, float (&acc)[2][MT]) const {
#pragma unroll
        for (int m = 0; m < MT; ++m)
            if (m < M) {
                const float g = acc[0][m], u = acc[1][m];
                a[(size_t)m * F + unit] = (g / (1.0f + __expf(-g))) * u;
            }
    }
};

template <typename WT, int MT, int D>
__global__ __launch_bounds__(WG_THREADS, 1) void k_gateup(GateUpOp<WT, MT> op, const float* __restrict__ h,
                                                          const float* __restrict__ gain, float eps) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    GemvPhase<WT, MT, D, GateUpOp<WT, MT>> ph;
    ph.setup(op.F, op.d, op.M, blockIdx.x, gridDim.x);
    ph.prefetch(op);
    ph.run(op, h, gain, eps, lds, lds + XS_BUDGET_BYTES / 4);
}

// ---- a7: final RMSNorm -> output projection -> fused arg-max -------------------------------------------
// Lane 63 of every wave keeps the running (max, lowest index) of the rows it produced; workgroups publish
// partials and the last one to finish reduces them (lowest index wins ties) and writes the token(s).
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
    __device__ __forceinline__ void wrows(int unit, const WT* (&r)[2]) const {
        r[0] = w + (size_t)(unit * 2) * d;
        r[1] = w + (size_t)min(unit * 2 + 1, V - 1) * d;
    }
    __device__ __forceinline__ void done(int unit, float (&acc)[2][MT]) {
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

template <typename WT, int MT, int D>
__global__ __launch_bounds__(WG_THREADS, 1) void k_head(const WT* __restrict__ w, const float* __restrict__ h,
                                                        const float* __restrict__ gain, float eps, int V, int d,
                                                        int M, HeadOut out, DevState* st) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* red = lds + XS_BUDGET_BYTES / 4;
    HeadOp<WT, MT> op;
    op.w = w; op.V = V; op.d = d; op.M = M; op.logits = out.logits;
#pragma unroll
    for (int m = 0; m < MT; ++m) { op.best_v[m] = -INFINITY; op.best_i[m] = 0x7FFFFFFF; }
    GemvPhase<WT, MT, D, HeadOp<WT, MT>> ph;
    ph.setup((V + 1) / 2, d, M, blockIdx.x, gridDim.x);
    ph.prefetch(op);
    ph.run(op, h, gain, eps, lds, red);

    // workgroup reduce of the per-wave bests (held by lane 63 of each wave)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __syncthreads();
    float* sv = lds;                                              // [NWAVE][MT]
    int* si = reinterpret_cast<int*>(lds + NWAVE * MAX_ROWS);     // [NWAVE][MT]
    if (lane == 63)
#pragma unroll
        for (int m = 0; m < MT; ++m) { sv[wave * MT + m] = op.best_v[m]; si[wave * MT + m] = op.best_i[m]; }
    __syncthreads();
    if (tid < M) {
        float bv = -INFINITY; int bi = 0x7FFFFFFF;
        for (int w2 = 0; w2 < NWAVE; ++w2) {
            const float v = sv[w2 * MT + tid]; const int i = si[w2 * MT + tid];
            if (better(v, i, bv, bi)) { bv = v; bi = i; }
        }
        out.part_val[(size_t)blockIdx.x * MAX_ROWS + tid] = bv;
        out.part_idx[(size_t)blockIdx.x * MAX_ROWS + tid] = bi;
    }
    __threadfence();
    __syncthreads();
    __shared__ unsigned s_last;
    if (tid == 0) s_last = (atomicAdd(out.counter, 1u) == gridDim.x - 1) ? 1u : 0u;
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    // final reduce: wave m handles row m; lanes stride over the workgroups' partials
    for (int m = wave; m < M; m += NWAVE) {
        float bv = -INFINITY; int bi = 0x7FFFFFFF;
        for (unsigned g = lane; g < gridDim.x; g += 64) {
            const float v = __builtin_nontemporal_load(out.part_val + (size_t)g * MAX_ROWS + m);
            const int i = __builtin_nontemporal_load(out.part_idx + (size_t)g * MAX_ROWS + m);
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
    if (tid == 0) *out.counter = 0u;
}

// ---- a3: causal attention of M rows over the contiguous cache, split along positions --------------------
// grid (n_splits_max, Hkv).  A workgroup handles one split of ATT_SL positions of one KV head for all rows
// and all query heads of the group.  K and V rows are read once, straight from the cache with coalesced
// row loads (lanes split head_dim), scores are reduced on the DPP network, soft-max statistics per split go
// to the workspace, and the last workgroup of a KV head to finish merges the splits in ascending order.
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

constexpr int ATT_PPW = ATT_SL / NWAVE;   // positions per wave per split (16)

// LDS: scores [ATT_QC][ATT_SL] + per-wave output partials [NWAVE][ATT_QC][hd] + (max, sum) [ATT_QC][2]
__host__ __device__ constexpr size_t attn_lds_bytes(int hd) {
    return sizeof(float) * (size_t)(ATT_QC * ATT_SL + NWAVE * ATT_QC * hd + 2 * ATT_QC);
}

// LPP = lanes per position = hd / 4 (each lane holds 4 consecutive dims of a K or V row)
template <typename WT, int LPP>
__device__ __forceinline__ void attn_split(const WT* __restrict__ kc, const WT* __restrict__ vc, const AttnArgs& a,
                                           float* lds, int split, int g) {
    constexpr int PPL = 64 / LPP;            // positions covered by one wave-wide row load
    constexpr int NL = ATT_PPW / PPL > 0 ? ATT_PPW / PPL : 1;   // row loads per wave per split
    static_assert(NL * PPL * NWAVE == ATT_SL || PPL > ATT_PPW, "split length must tile");
    const int hd = a.L.hd, H = a.L.H, Hkv = a.L.Hkv, grp = H / Hkv, M = a.rows.M;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pos0 = row_pos(a.rows, a.st, 0);
    const int Ltot = pos0 + M;
    const int n_active = (Ltot + ATT_SL - 1) / ATT_SL;
    const int start = split * ATT_SL, npos = min(ATT_SL, Ltot - start);
    float* sc = lds;                               // [ATT_QC][ATT_SL]
    float* ored = sc + ATT_QC * ATT_SL;            // [NWAVE][ATT_QC][hd]
    float* mls = ored + NWAVE * ATT_QC * hd;       // [ATT_QC][2]
    const float scale = 1.0f / sqrtf((float)hd);
    const int sub = lane / LPP, dl = (lane % LPP) * 4;   // position slot inside a row load, first dim of the lane

    // positions owned by this wave: j = (l * NWAVE + wave) * PPL + sub  (interleaved over waves)
    float kf[NL][4], vf[NL][4];
#pragma unroll
    for (int l = 0; l < NL; ++l) {
        const int j = (l * NWAVE + wave) * PPL + sub;
#pragma unroll
        for (int e = 0; e < 4; ++e) { kf[l][e] = 0.f; vf[l][e] = 0.f; }
        if (j < npos) {
            const WT* kr = kc + ((size_t)g * a.L.max_seq + start + j) * hd + dl;
            const WT* vr = vc + ((size_t)g * a.L.max_seq + start + j) * hd + dl;
            if (sizeof(WT) == 2) {
                const u32x2 kk = *reinterpret_cast<const u32x2*>(kr), vv = *reinterpret_cast<const u32x2*>(vr);
                kf[l][0] = __uint_as_float(kk.x << 16); kf[l][1] = __uint_as_float(kk.x & 0xFFFF0000u);
                kf[l][2] = __uint_as_float(kk.y << 16); kf[l][3] = __uint_as_float(kk.y & 0xFFFF0000u);
                vf[l][0] = __uint_as_float(vv.x << 16); vf[l][1] = __uint_as_float(vv.x & 0xFFFF0000u);
                vf[l][2] = __uint_as_float(vv.y << 16); vf[l][3] = __uint_as_float(vv.y & 0xFFFF0000u);
            } else {
                const f32x4 kk = *reinterpret_cast<const f32x4*>(kr), vv = *reinterpret_cast<const f32x4*>(vr);
                kf[l][0] = kk.x; kf[l][1] = kk.y; kf[l][2] = kk.z; kf[l][3] = kk.w;
                vf[l][0] = vv.x; vf[l][1] = vv.y; vf[l][2] = vv.z; vf[l][3] = vv.w;
            }
        }
    }
    const int nq = M * grp;   // query vectors: qi = m * grp + gi
    for (int q0 = 0; q0 < nq; q0 += ATT_QC) {
        const int nqc = min(ATT_QC, nq - q0);
        // scores: the lane group of a position reduces its 4-dim partial dot products on the DPP network
        for (int ql = 0; ql < nqc; ++ql) {
            const int qi = q0 + ql, m = qi / grp, hq = g * grp + (qi - m * grp);
            const f32x4 qv = *reinterpret_cast<const f32x4*>(a.q + (size_t)m * H * hd + (size_t)hq * hd + dl);
#pragma unroll
            for (int l = 0; l < NL; ++l) {
                float s = kf[l][0] * qv.x;
                s = fmaf(kf[l][1], qv.y, s); s = fmaf(kf[l][2], qv.z, s); s = fmaf(kf[l][3], qv.w, s);
                s = group_sum_dpp<LPP>(s);
                const int j = (l * NWAVE + wave) * PPL + sub;
                if ((lane % LPP) == LPP - 1 && j < ATT_SL)
                    sc[ql * ATT_SL + j] = (j < npos && start + j <= pos0 + m) ? s * scale : -INFINITY;
            }
        }
        __syncthreads();
        // soft-max statistics per query (one wave per query); probabilities written back in place
        for (int ql = wave; ql < nqc; ql += NWAVE) {
            const float s0 = sc[ql * ATT_SL + lane], s1 = sc[ql * ATT_SL + 64 + lane];
            const float mx = wave_max(fmaxf(s0, s1));
            float p0 = 0.f, p1 = 0.f;
            if (mx > -INFINITY) { p0 = __expf(s0 - mx); p1 = __expf(s1 - mx); }
            sc[ql * ATT_SL + lane] = p0; sc[ql * ATT_SL + 64 + lane] = p1;
            const float l = wave_sum(p0 + p1);
            if (lane == 0) { mls[ql * 2] = mx; mls[ql * 2 + 1] = l; }
        }
        __syncthreads();
        // o[dims of this lane] += p[j] * V[j][dims] over this wave's positions, then over the position slots
        for (int ql = 0; ql < nqc; ++ql) {
            float o[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int l = 0; l < NL; ++l) {
                const int j = (l * NWAVE + wave) * PPL + sub;
                const float p = j < ATT_SL ? sc[ql * ATT_SL + j] : 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = fmaf(p, vf[l][e], o[e]);
            }
            // fold the PPL position slots of the wave (lanes with equal lane % LPP) in a fixed order
#pragma unroll
            for (int off = LPP; off < 64; off <<= 1)
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] += __shfl_xor(o[e], off);
            if (sub == 0)
                *reinterpret_cast<f32x4*>(ored + ((size_t)wave * ATT_QC + ql) * hd + dl) = f32x4{o[0], o[1], o[2], o[3]};
        }
        __syncthreads();
        for (int idx = tid; idx < nqc * hd; idx += WG_THREADS) {
            const int ql = idx / hd, dim = idx - ql * hd;
            float o = 0.f;
#pragma unroll
            for (int w = 0; w < NWAVE; ++w) o += ored[((size_t)w * ATT_QC + ql) * hd + dim];
            const int qi = q0 + ql, m = qi / grp, hq = g * grp + (qi - m * grp);
            a.part_o[(((size_t)split * MAX_ROWS + m) * H + hq) * hd + dim] = o;
            if (dim == 0) {
                float* ml = a.part_ml + (((size_t)split * MAX_ROWS + m) * H + hq) * 2;
                ml[0] = mls[ql * 2]; ml[1] = mls[ql * 2 + 1];
            }
        }
        __syncthreads();
    }
    // last workgroup of this KV head merges the splits
    __threadfence();
    __syncthreads();
    __shared__ unsigned s_last;
    if (tid == 0) s_last = (atomicAdd(a.counters + g, 1u) == (unsigned)(n_active - 1)) ? 1u : 0u;
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    for (int idx = tid; idx < nq * hd; idx += WG_THREADS) {
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

template <typename WT>
__global__ __launch_bounds__(WG_THREADS, 1) void k_attn(const WT* __restrict__ kc, const WT* __restrict__ vc, AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int split = blockIdx.x, g = blockIdx.y;
    const int Ltot = row_pos(a.rows, a.st, 0) + a.rows.M;
    if (split * ATT_SL >= Ltot) return;
    switch (a.L.hd) {
        case 8: attn_split<WT, 2>(kc, vc, a, lds, split, g); break;
        case 16: attn_split<WT, 4>(kc, vc, a, lds, split, g); break;
        case 32: attn_split<WT, 8>(kc, vc, a, lds, split, g); break;
        case 64: attn_split<WT, 16>(kc, vc, a, lds, split, g); break;
        case 128: attn_split<WT, 32>(kc, vc, a, lds, split, g); break;
        default: attn_split<WT, 64>(kc, vc, a, lds, split, g); break;   // 256
    }
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
