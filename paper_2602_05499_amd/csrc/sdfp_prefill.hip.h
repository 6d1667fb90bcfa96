// The prompt's forward as matrix-matrix products ("given input x", paper Sec. II-A; the target forward that fills the
// cache before the first speculative step).  A prompt of hundreds of rows is bound by the matrix cores, not by the HBM
// read of the weights, so it does not go through the weight-streaming kernel 16 rows at a time (which re-reads every
// weight per 16 rows) but through a tiled GEMM per projection whose weights leave HBM once per panel of up to 512 rows
// (the workgroups that share a weight tile sit on one XCD and find it in that XCD's L2).  The same GEMM with a plain
// epilogue (PF_PLAIN) serves the products of the FIT pass (sdfp_fit.hip.h).
//
// What it must preserve: the cache rows and the residual stream it produces are the ones the decode kernels would
// produce, bit for bit (a rolled-back cache equals a freshly prefilled one; row i of a prompt equals the one-row decode
// of the same prefix).  So every output is computed with the arithmetic of sdfp_stream.hip.h:
//   * the reduction dimension is cut into NSHARE = 8 interleaved shares (share p owns the 4 consecutive 64-byte steps
//     4p .. 4p+3 of every 2 KB block of a weight row); a share's partial sum is one chain of
//     v_mfma_f32_16x16x32_bf16 accumulations over its steps in ascending order, three per step (the three bfloat16
//     pieces of the float32 activation, in order), weights as the A operand, activations as the B operand;
//   * the output is ((((0 + P0) + P1) + ...) + P7) in float32;
//   * norm scale, rotary embedding, SwiGLU, residual add, bfloat16 rounding of keys / values, the sum of squares of a
//     row and the split of an activation into pieces use the shared helpers of sdfp_common.hip.h, built from single
//     float32 operations that the compiler cannot contract with their neighbours;
//   * attention runs the decode kernels' own attn_split on 16-row chunks.
// The GEMM therefore walks the reduction dimension share by share (a permutation of the usual order), which costs
// nothing: every step of it is still a whole 64-byte line of 16 weight rows.
//
// Layout of a panel of P prompt rows in the workspace: h [P][d] float32 residual stream (updated in place); xs
// [3][P][Kx] bfloat16, the three pieces of the current projection input; q, att [P][H*hd] float32; rs [P] float32.
#pragma once
#include "sdfp_attn.hip.h"

namespace sdfp {

constexpr int PF_NSHARE = 8;             // shares of the reduction dimension (= waves of the decode kernels)
constexpr int PF_STEP_BYTES = 64;        // bytes of a weight row per matrix-core step (32 bfloat16)
constexpr int PF_SPS = 4;                // consecutive steps of a share per block
constexpr int PF_BLOCK_BYTES = PF_NSHARE * PF_SPS * PF_STEP_BYTES;   // 2 KB
constexpr int PF_TM = 64;                // prompt rows per workgroup tile
constexpr int PF_SLAB_ROW = PF_SPS * PF_STEP_BYTES + 16;   // staged bytes per (piece, prompt row) of a slab, padded: 272
constexpr int PF_SLAB_BYTES = 3 * PF_TM * PF_SLAB_ROW;     // 52224
constexpr int PF_LDS_BYTES = 2 * PF_SLAB_BYTES;            // double-buffered

enum { PF_QKV = 0, PF_OPROJ = 1, PF_GATEUP = 2, PF_DOWN = 3, PF_PLAIN = 4 };   // PF_PLAIN: out = (out +) x W^T, nothing fused

struct PfGemm {
    const bf16_t* w[3];      // QKV: wq wk wv; gate/up: w_gate w_up; else the matrix in w[0]; row-major [N][Kd]
    const bf16_t* xs;        // [3][P][Kd] pieces of the input rows
    size_t xs_piece;         // elements between pieces (P * Kd)
    int Kd;                  // reduction length
    int n_tiles;             // 16-row weight tiles of the projection
    int M;                   // valid prompt rows of the panel
    int pos0;                // absolute position of the panel's row 0
    const float* rs;         // [P] reciprocal RMS of the input rows (QKV, gate/up), else nullptr
    float* h;                // O / down: residual stream [P][d], updated in place
    float* q;                // QKV: queries [P][H*hd]
    bf16_t *kc, *vc;         // QKV: this layer's key / value planes [Hkv][max_seq][hd]
    bf16_t* xs_out;          // gate/up: [3][P][F] pieces of the feed-forward activation
    size_t xs_out_piece;
    const float *cosT, *sinT;
    float* out;              // PF_PLAIN: [M][ldo] float32 result
    int ldo;                 // PF_PLAIN: elements between rows of out
    int accumulate;          // PF_PLAIN: add to what out holds instead of overwriting it
    float* part;             // O / down dealt by shares: [8][P][d] partial sums
    size_t part_arr;         // floats per array of part (P * d)
    int n_nt;                // groups of 8 * NT weight tiles
    int my;                  // row tiles of the panel (64 rows each)
    int n_groups;            // workgroups that share a tile's reduction dimension: 1, 2, 4 or 8
    LayerDims L;
};

// ---- RMSNorm prologue of a projection: sum of squares of a row in the decode kernels' order, the row times the gain
// split into pieces.  One workgroup of 512 threads per prompt row; threads 0..447 are the decode kernels' staging
// threads: thread t adds the 8-value chunks t, t + 448, ... in ascending order, lanes are folded by the DPP tree, the
// eight wave sums are added in wave order (the last wave's is 0). -----------------------------------------------------
__global__ __launch_bounds__(512) void k_pf_norm_split(const float* __restrict__ h, const float* __restrict__ gain, int d,
                                                       float eps, float* __restrict__ rs, bf16_t* __restrict__ xs,
                                                       size_t xs_piece) {
    __shared__ float ss[NWAVE];
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* row = h + (size_t)m * d;
    const int nchunk = d >> 3;
    float s = 0.f;
    for (int c = tid; c < nchunk && wave != NWAVE - 1; c += WG_THREADS - 64) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(row + c * 8), b = *reinterpret_cast<const f32x4*>(row + c * 8 + 4);
        s = add_rn(s, sq8(a, b));
        const f32x4 g0 = *reinterpret_cast<const f32x4*>(gain + c * 8), g1 = *reinterpret_cast<const f32x4*>(gain + c * 8 + 4);
        const float x[8] = {mul_rn(a.x, g0.x), mul_rn(a.y, g0.y), mul_rn(a.z, g0.z), mul_rn(a.w, g0.w),
                            mul_rn(b.x, g1.x), mul_rn(b.y, g1.y), mul_rn(b.z, g1.z), mul_rn(b.w, g1.w)};
        u32x4 piece[3];
        split3_bf16(x, piece);
#pragma unroll
        for (int p = 0; p < 3; ++p) *reinterpret_cast<u32x4*>(xs + p * xs_piece + (size_t)m * d + c * 8) = piece[p];
    }
    s = wave_sum_last(s);
    if (lane == 63) ss[wave] = s;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < NWAVE; ++w) t = add_rn(t, ss[w]);
        rs[m] = rms_recip(t, d, eps);
    }
}

// rows without a norm (the attention output in front of the O projection): pieces only
__global__ __launch_bounds__(256) void k_pf_split(const float* __restrict__ x, int n8, bf16_t* __restrict__ xs, size_t xs_piece) {
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n8; c += gridDim.x * blockDim.x) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(x + (size_t)c * 8), b = *reinterpret_cast<const f32x4*>(x + (size_t)c * 8 + 4);
        const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        u32x4 piece[3];
        split3_bf16(v, piece);
#pragma unroll
        for (int p = 0; p < 3; ++p) *reinterpret_cast<u32x4*>(xs + p * xs_piece + (size_t)c * 8) = piece[p];
    }
}

// embedding rows of a panel: h[m][:] = tok_emb[prompt[m]][:]
__global__ __launch_bounds__(256) void k_pf_embed(const int* __restrict__ prompt, const bf16_t* __restrict__ emb, int d, int V,
                                                  float* __restrict__ h) {
    const int m = blockIdx.x;
    const int tok = min(max(prompt[m], 0), V - 1);
    for (int k = threadIdx.x * 4; k < d; k += blockDim.x * 4) {
        const u32x2 r = *reinterpret_cast<const u32x2*>(emb + (size_t)tok * d + k);
        *reinterpret_cast<f32x4*>(h + (size_t)m * d + k) =
            f32x4{__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u), __uint_as_float(r.y << 16),
                  __uint_as_float(r.y & 0xFFFF0000u)};
    }
}

// ---- the GEMM.  A workgroup computes 8 * NT weight tiles (128 * NT output rows) x PF_TM prompt rows; wave w owns the NT
// weight tiles w * NT .. and all four 16-row column tiles, so a weight is read by one wave only and an input piece read
// from LDS feeds NT matrix-core instructions.  Weights go from memory straight into the A operand (lane l: row l % 16,
// bytes (l / 16) * 16 .. of the step, as in the decode kernels), one slab ahead; the input pieces of a slab -- the 4 steps
// that one share owns in one block, for all 64 prompt rows -- are staged in LDS, double-buffered, and read as the B
// operand (lane l: prompt row l % 16, the same bytes of the step).
//
// Workgroups that read the same weights (the panel's row tiles of one weight tile group) are neighbours on one XCD,
// so the weights come from HBM once and from that XCD's L2 afterwards: workgroup id -> XCD id % 8, place id / 8 on it;
// a place is (column c = (tile group, share group), row tile), row tile fastest; column c lives on XCD c % 8.
//
// PARTIAL: the projection is too narrow to fill the chip with whole outputs (O and down projections), so the shares of
// the reduction dimension are dealt to n_groups workgroups per tile; each writes its shares' partial sums P_p to
// part[p][row][N], and k_pf_residual adds them in share order.
template <int KIND, int NT, bool PARTIAL>
__global__ __launch_bounds__(WG_THREADS, 1) void k_pf_gemm(PfGemm a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, gq = lane >> 4;
    const int xcd = blockIdx.x & 7, place = blockIdx.x >> 3;
    const int col = (place / a.my) * 8 + xcd;
    if (col >= a.n_nt * a.n_groups) return;                 // uniform over the workgroup
    const int grp = col % a.n_groups;
    const int m0 = (place % a.my) * PF_TM;                  // first prompt row of the workgroup tile
    const int t0 = (col / a.n_groups) * (8 * NT) + wave * NT;   // the wave's first weight tile
    const int pitch = a.Kd * 2;                             // bytes per weight row
    const int S = pitch / PF_STEP_BYTES;                    // steps per weight row
    const int nblk = (S + PF_NSHARE * PF_SPS - 1) / (PF_NSHARE * PF_SPS);
    const int hd = a.L.hd, H = a.L.H, Hkv = a.L.Hkv, half = hd >> 1, tph = hd >> 4;

    // this lane's weight row of tile t (tiles past the end repeat the last one; their outputs are dropped)
    auto row_ptr = [&](int t) -> const char* {
        t = min(t, a.n_tiles - 1);
        const bool hi = r16 >= 8;
        if (KIND == PF_QKV) {          // tile = 8 rotary pairs of one head of wq, wk or wv: rows (i, i + hd / 2)
            const int hs = t / tph, jj = t - hs * tph;
            const int sel = hs < H ? 0 : (hs < H + Hkv ? 1 : 2);
            const int head = hs - (sel == 0 ? 0 : (sel == 1 ? H : H + Hkv));
            const int row = head * hd + jj * 8 + (r16 & 7) + (hi ? half : 0);
            return (const char*)a.w[sel] + (size_t)row * pitch + gq * 16;
        }
        if (KIND == PF_GATEUP)         // tile = 8 gate rows and the 8 up rows of the same units
            return (const char*)a.w[hi ? 1 : 0] + (size_t)(t * 8 + (r16 & 7)) * pitch + gq * 16;
        return (const char*)a.w[0] + (size_t)(t * 16 + r16) * pitch + gq * 16;
    };
    const char* wrow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) wrow[t] = row_ptr(t0 + t);

    // staging of a slab: 3 pieces x 64 prompt rows x 256 bytes = 3072 16-byte units, 6 per thread
    const char* xs_base = (const char*)a.xs;
    auto slab_dst = [&](int u, int buf) -> char* {
        const int unit = tid + u * WG_THREADS;
        const int piece = unit >> 10, row = (unit >> 4) & 63, part = unit & 15;
        return lds + buf * PF_SLAB_BYTES + (piece * PF_TM + row) * PF_SLAB_ROW + part * 16;
    };
    // slab i of the walk: share p = i / nblk, block b = i % nblk; its first byte in a row, and how many of its 4 steps exist
    auto slab_byte0 = [&](int i) { return (i % nblk) * PF_BLOCK_BYTES + (i / nblk) * (PF_SPS * PF_STEP_BYTES); };
    auto slab_steps = [&](int i) { return max(0, min(PF_SPS, S - ((i % nblk) * (PF_NSHARE * PF_SPS) + (i / nblk) * PF_SPS))); };
    const int spg = PF_NSHARE / a.n_groups;                 // shares per group
    const int i_lo = grp * spg * nblk, i_hi = i_lo + spg * nblk;

    f32x4 total[PARTIAL ? 1 : NT][PARTIAL ? 1 : 4], acc[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (!PARTIAL) total[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    // Every load of the loop below is unconditional and its address clamped into the row: a load under a condition makes
    // the compiler wait, at the join, for everything in flight, and the pipeline (pieces and weights one slab ahead)
    // would stall once per step.  What a clamped load brings is never used: the steps a slab does not have are skipped.
    u32x4 stage[6];
    u32x4 wa[NT][PF_SPS];   // the wave's weight steps: of this slab until a step is multiplied, of the next one after
    const int last16 = pitch - 16, last_step = pitch - PF_STEP_BYTES;
    auto load_slab = [&](int i) {
        const int byte0 = slab_byte0(i);
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            const int unit = tid + u * WG_THREADS;              // unit = (piece * 64 + row) * 16 + sixteenth
            const int piece = unit >> 10, row = (unit >> 4) & 63, part = unit & 15;
            const int m = min(m0 + row, a.M - 1);
            stage[u] = *reinterpret_cast<const u32x4*>(xs_base + ((size_t)piece * a.xs_piece + (size_t)m * a.Kd) * 2 +
                                                       min(byte0 + part * 16, last16));
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 6; ++u) *reinterpret_cast<u32x4*>(slab_dst(u, buf)) = stage[u];
    };
    auto load_weight_step = [&](int byte0, int s) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
            wa[t][s] = *reinterpret_cast<const u32x4*>(wrow[t] + min(byte0 + s * PF_STEP_BYTES, last_step));
    };

    load_slab(i_lo);
    store_slab(0);
#pragma unroll
    for (int s = 0; s < PF_SPS; ++s) load_weight_step(slab_byte0(i_lo), s);
    __syncthreads();
    for (int i = i_lo; i < i_hi; ++i) {
        const int buf = (i - i_lo) & 1;
        const int nst = slab_steps(i);
        const int i_next = min(i + 1, i_hi - 1);               // the last slab fetches itself again, unused
        const int byte0_next = slab_byte0(i_next);
        load_slab(i_next);                                     // the next slab's pieces travel while this one is multiplied
        const char* xb = lds + buf * PF_SLAB_BYTES + r16 * PF_SLAB_ROW + gq * 16;
#pragma unroll
        for (int s = 0; s < PF_SPS; ++s) {
            if (s < nst) {   // uniform over the workgroup; LDS reads and matrix-core steps only
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    u32x4 xb3[3];
#pragma unroll
                    for (int p = 0; p < 3; ++p)
                        xb3[p] = *reinterpret_cast<const u32x4*>(xb + (p * PF_TM + j * 16) * PF_SLAB_ROW + s * PF_STEP_BYTES);
                    // every accumulator sees its three pieces in order; neighbours in the instruction stream are independent
#pragma unroll
                    for (int p = 0; p < 3; ++p)
#pragma unroll
                        for (int t = 0; t < NT; ++t)
                            acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(bf16x8, wa[t][s]), __builtin_bit_cast(bf16x8, xb3[p]), acc[t][j], 0, 0, 0);
                }
            }
            load_weight_step(byte0_next, s);                  // this step's registers are free: the next slab's weights
        }
        if ((i + 1) % nblk == 0) {   // the share's partial sums are complete
            const int p = i / nblk;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (PARTIAL) {
                        const int tile = t0 + t, m = m0 + j * 16 + r16;
                        if (tile < a.n_tiles && m < a.M)
                            *reinterpret_cast<f32x4*>(a.part + (size_t)p * a.part_arr + (size_t)m * a.L.d + tile * 16 + gq * 4) = acc[t][j];
                    } else {     // added in share order
                        f32x4& T = total[PARTIAL ? 0 : t][PARTIAL ? 0 : j];
                        T.x = add_rn(T.x, acc[t][j].x); T.y = add_rn(T.y, acc[t][j].y);
                        T.z = add_rn(T.z, acc[t][j].z); T.w = add_rn(T.w, acc[t][j].w);
                    }
                    acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
        }
        store_slab(buf ^ 1);                                   // the other buffer's last readers passed the barrier below
        __syncthreads();
    }
    if (PARTIAL) return;

    // ---- epilogue.  Lane l holds, per tile, prompt row (column) l % 16 and output rows 4 * (l / 16) .. + 3 of the tile.
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tile = t0 + t;
        if (tile >= a.n_tiles) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + j * 16 + r16;
            f32x4 v = total[PARTIAL ? 0 : t][PARTIAL ? 0 : j];
            if (KIND == PF_PLAIN) {
                if (m < a.M) {
                    float* o = a.out + (size_t)m * a.ldo + tile * 16 + gq * 4;
                    if (a.accumulate) {
                        const f32x4 r = *reinterpret_cast<const f32x4*>(o);
                        v = f32x4{add_rn(r.x, v.x), add_rn(r.y, v.y), add_rn(r.z, v.z), add_rn(r.w, v.w)};
                    }
                    *reinterpret_cast<f32x4*>(o) = v;
                }
                continue;
            }
            if (KIND == PF_OPROJ || KIND == PF_DOWN) {
                if (m < a.M) {
                    float* o = a.h + (size_t)m * a.L.d + tile * 16 + gq * 4;
                    const f32x4 r = *reinterpret_cast<const f32x4*>(o);
                    *reinterpret_cast<f32x4*>(o) = f32x4{add_rn(r.x, v.x), add_rn(r.y, v.y), add_rn(r.z, v.z), add_rn(r.w, v.w)};
                }
                continue;
            }
            // QKV, gate/up: rows r and r + 8 of the tile form a pair; they sit in lanes l and l + 32
            const float rsm = a.rs[min(m, a.M - 1)];
            v = f32x4{mul_rn(v.x, rsm), mul_rn(v.y, rsm), mul_rn(v.z, rsm), mul_rn(v.w, rsm)};
            f32x4 o2;
            o2.x = __shfl_xor(v.x, 32); o2.y = __shfl_xor(v.y, 32); o2.z = __shfl_xor(v.z, 32); o2.w = __shfl_xor(v.w, 32);
            if (gq >= 2 || m >= a.M) continue;          // lanes 0..31 hold rows 0..7 (first of each pair)
            float lo[4] = {v.x, v.y, v.z, v.w}, hi[4] = {o2.x, o2.y, o2.z, o2.w};
            if (KIND == PF_GATEUP) {
                const int u = tile * 8 + gq * 4;        // units u .. u + 3 of prompt row m
                float act[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) act[e] = swiglu(lo[e], hi[e]);
                // pieces of 4 consecutive values (the split works on 8; the upper 4 are zeros and are not stored)
                const float x8[8] = {act[0], act[1], act[2], act[3], 0.f, 0.f, 0.f, 0.f};
                u32x4 piece[3];
                split3_bf16(x8, piece);
#pragma unroll
                for (int p = 0; p < 3; ++p)
                    *reinterpret_cast<u32x2*>(a.xs_out + p * a.xs_out_piece + (size_t)m * a.L.F + u) = u32x2{piece[p].x, piece[p].y};
            } else {   // QKV
                const int hs = tile / tph, i0 = (tile - hs * tph) * 8 + gq * 4;   // dims i0 .. i0 + 3 and + half
                const int pos = a.pos0 + m;
                if (hs < H + Hkv) {
                    const f32x4 c = *reinterpret_cast<const f32x4*>(a.cosT + (size_t)pos * half + i0);
                    const f32x4 sn = *reinterpret_cast<const f32x4*>(a.sinT + (size_t)pos * half + i0);
                    rotary_pair(lo[0], hi[0], c.x, sn.x); rotary_pair(lo[1], hi[1], c.y, sn.y);
                    rotary_pair(lo[2], hi[2], c.z, sn.z); rotary_pair(lo[3], hi[3], c.w, sn.w);
                }
                if (hs < H) {
                    float* o = a.q + (size_t)m * H * hd + (size_t)hs * hd + i0;
                    *reinterpret_cast<f32x4*>(o) = f32x4{lo[0], lo[1], lo[2], lo[3]};
                    *reinterpret_cast<f32x4*>(o + half) = f32x4{hi[0], hi[1], hi[2], hi[3]};
                } else {
                    const bool isk = hs < H + Hkv;
                    const int kvh = isk ? hs - H : hs - H - Hkv;
                    bf16_t* o = (isk ? a.kc : a.vc) + ((size_t)kvh * a.L.max_seq + pos) * hd + i0;
                    *reinterpret_cast<u32x2*>(o) = u32x2{(unsigned)f32_to_bf16(lo[0]) | ((unsigned)f32_to_bf16(lo[1]) << 16),
                                                         (unsigned)f32_to_bf16(lo[2]) | ((unsigned)f32_to_bf16(lo[3]) << 16)};
                    *reinterpret_cast<u32x2*>(o + half) = u32x2{(unsigned)f32_to_bf16(hi[0]) | ((unsigned)f32_to_bf16(hi[1]) << 16),
                                                                (unsigned)f32_to_bf16(hi[2]) | ((unsigned)f32_to_bf16(hi[3]) << 16)};
                }
            }
        }
    }
}


// O / down projection in PARTIAL form: h[m][n] += ((((0 + P0) + P1) + ...) + P7), 4 outputs per thread
__global__ __launch_bounds__(256) void k_pf_residual(float* __restrict__ h, const float* __restrict__ part, size_t part_arr, int n4) {
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n4; c += gridDim.x * blockDim.x) {
        f32x4 t = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < PF_NSHARE; ++p) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(part + (size_t)p * part_arr + (size_t)c * 4);
            t = f32x4{add_rn(t.x, v.x), add_rn(t.y, v.y), add_rn(t.z, v.z), add_rn(t.w, v.w)};
        }
        const f32x4 r = *reinterpret_cast<const f32x4*>(h + (size_t)c * 4);
        *reinterpret_cast<f32x4*>(h + (size_t)c * 4) = f32x4{add_rn(r.x, t.x), add_rn(r.y, t.y), add_rn(r.z, t.z), add_rn(r.w, t.w)};
    }
}

// ---- attention of a panel: the decode kernels' attn_split on 16-row chunks.  A workgroup takes (chunk, KV head) items
// and runs the chunk's splits one after another into a region of its own (split partials, merge counter), so that the
// last call merges them in ascending split order exactly as the last workgroup of a KV head does in the forward kernel.
struct PfAttn {
    const float* q;        // [P][H*hd] of the panel
    float* att;            // [P][H*hd]
    const bf16_t *kc, *vc; // this layer's planes
    float* part;           // per workgroup: part_o [n_splits][16][grp][hd] then part_ml [n_splits][16][grp][2]
    size_t part_stride;    // floats per workgroup region
    size_t part_ml_off;    // floats from a region's start to its part_ml
    unsigned* counters;    // one per workgroup, left at 0
    int M;                 // valid rows of the panel
    int pos0;              // absolute position of the panel's row 0
    LayerDims L;
};
template <int LPP>
__global__ __launch_bounds__(WG_THREADS, 1) void k_pf_attn(PfAttn a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int grp = a.L.H / a.L.Hkv;
    const int n_chunks = (a.M + MAX_ROWS - 1) / MAX_ROWS;
    AttnArgs aa;
    aa.part_o = a.part + (size_t)blockIdx.x * a.part_stride;
    aa.part_ml = aa.part_o + a.part_ml_off;
    aa.counters = a.counters + blockIdx.x;
    aa.part_H = grp;
    aa.L = a.L; aa.st = nullptr;
    for (int it = blockIdx.x; it < n_chunks * a.L.Hkv; it += gridDim.x) {
        const int c = it / a.L.Hkv, g = it - c * a.L.Hkv;
        aa.q = a.q + (size_t)c * MAX_ROWS * a.L.H * a.L.hd;
        aa.att = a.att + (size_t)c * MAX_ROWS * a.L.H * a.L.hd;
        aa.rows = Rows{min(MAX_ROWS, a.M - c * MAX_ROWS), ROWS_PROMPT, a.pos0 + c * MAX_ROWS};
        aa.part_h0 = g * grp;
        const int n_active = (aa.rows.off + aa.rows.M + ATT_SL - 1) / ATT_SL;
        for (int split = 0; split < n_active; ++split) {
            attn_split<bf16_t, LPP, 0, true>(a.kc, a.vc, aa, reinterpret_cast<float*>(lds), split, g);
            __syncthreads();
        }
    }
}

}  // namespace sdfp
