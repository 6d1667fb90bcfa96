// FIT layer scores (paper Sec. III-B, Eq. 11; Alg. 1 Stage A): T_l = 1/N sum_i || grad_{theta_l} f(z_i, theta) ||^2,
// f = mean next-token cross-entropy of a calibration sequence.  One forward over the whole sequence that keeps what
// the backward needs, one backward, and the squared norm of every layer tensor's gradient -- without ever forming a
// weight gradient: for y = x W^T over T positions, grad W = dY^T X and
//     || dY^T X ||_F^2 = sum_{t,t'} (dY_t . dY_t') (X_t . X_t'),
// the sum over the entrywise product of two T x T Gram matrices (T <= 2048 here, the matrices have 10^7..10^8 entries).
//
// Arithmetic: weights are the stored bfloat16 values, every activation and gradient is float32.  Products with a weight
// matrix (forward, and backward with respect to the input through a transposed copy of the matrix) run through the
// prompt path's matrix-core GEMM (sdfp_prefill.hip.h: float32 activations as three bfloat16 pieces, float32
// accumulation); Gram matrices through the float32 matrix-core instruction; attention, norms, rotary embedding, SwiGLU
// and the cross-entropy on the vector ALUs.  Keys and values are not rounded: there is no cache in this pass.
#pragma once
#include "sdfp_prefill.hip.h"

namespace sdfp {

constexpr int FIT_MAX_T = 2048;   // positions per calibration sequence (an attention row of probabilities is kept in LDS)
constexpr int FIT_GRAM_SLICES = 32;   // most stretches the reduction dimension of a Gram matrix is cut into

__device__ __forceinline__ float fit_wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
// sum over a workgroup of up to 16 waves; sh: 16 floats of LDS; every thread gets the sum
__device__ __forceinline__ float fit_block_sum(float v, float* sh) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = fit_wave_sum(v);
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    float s = 0.f;
    for (int w = 0; w < nw; ++w) s += sh[w];
    return s;
}
__device__ __forceinline__ float fit_block_max(float v, float* sh) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_max(v);
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    float s = sh[0];
    for (int w = 1; w < nw; ++w) s = fmaxf(s, sh[w]);
    return s;
}

// ---- RMSNorm forward: y = x * rs * gain, rs = (mean(x^2) + eps)^(-1/2); one workgroup per row -------------------------
__global__ __launch_bounds__(256) void k_fit_rmsnorm(const float* __restrict__ x, const float* __restrict__ gain, int d, float eps,
                                                     float* __restrict__ y, float* __restrict__ rs) {
    __shared__ float sh[16];
    const float* row = x + (size_t)blockIdx.x * d;
    float s = 0.f;
    for (int c = threadIdx.x; c < d; c += blockDim.x) s += row[c] * row[c];
    s = fit_block_sum(s, sh);
    const float r = 1.0f / sqrtf(s / (float)d + eps);
    if (threadIdx.x == 0) rs[blockIdx.x] = r;
    for (int c = threadIdx.x; c < d; c += blockDim.x) y[(size_t)blockIdx.x * d + c] = row[c] * r * gain[c];
}
// RMSNorm backward with respect to the input, added to a residual gradient: out = res + dx,
// dx = gain dy rs - x rs^3 (sum_c gain dy x) / d.  out may be res.
__global__ __launch_bounds__(256) void k_fit_rmsnorm_bwd(const float* __restrict__ x, const float* __restrict__ gain,
                                                         const float* __restrict__ rs, const float* __restrict__ dy, int d,
                                                         const float* res, float* out) {
    __shared__ float sh[16];
    const size_t o = (size_t)blockIdx.x * d;
    float s = 0.f;
    for (int c = threadIdx.x; c < d; c += blockDim.x) s += gain[c] * dy[o + c] * x[o + c];
    s = fit_block_sum(s, sh);
    const float r = rs[blockIdx.x], k = r * r * r * s / (float)d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        const float dx = gain[c] * dy[o + c] * r - x[o + c] * k;
        out[o + c] = (res ? res[o + c] : 0.f) + dx;
    }
}
// squared norm of the gain's gradient, dgain_c = sum_t dy[t][c] x[t][c] rs[t], added to *acc.  A workgroup of 1024 threads
// takes 64 columns: thread (column cx, row group ry) adds the rows ry, ry + 16, ..., the 16 groups meet in LDS.
__global__ __launch_bounds__(1024) void k_fit_dgain_sumsq(const float* __restrict__ x, const float* __restrict__ rs,
                                                          const float* __restrict__ dy, int T, int d, double* acc) {
    __shared__ float part[16][64];
    __shared__ float sh[16];
    const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6, c = blockIdx.x * 64 + cx;
    float g = 0.f;
    if (c < d)
        for (int t = ry; t < T; t += 16) g += dy[(size_t)t * d + c] * x[(size_t)t * d + c] * rs[t];
    part[ry][cx] = g;
    __syncthreads();
    float sq = 0.f;
    if (ry == 0) {
        float tot = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) tot += part[r][cx];
        sq = tot * tot;
    }
    const float s = fit_block_sum(sq, sh);
    if (threadIdx.x == 0) atomicAdd(acc, (double)s);
}

// ---- rotary embedding of [T][heads * hd] in place, pairs (i, i + hd/2); inverse: by minus the angle ---------------------
__global__ __launch_bounds__(256) void k_fit_rope(float* __restrict__ x, int heads, int hd, const float* __restrict__ cosT,
                                                  const float* __restrict__ sinT, int inverse) {
    const int t = blockIdx.x, half = hd >> 1;
    for (int e = threadIdx.x; e < heads * half; e += blockDim.x) {
        const int h = e / half, i = e - h * half;
        float* p = x + (size_t)t * heads * hd + (size_t)h * hd + i;
        const float c = cosT[(size_t)t * half + i], s = inverse ? -sinT[(size_t)t * half + i] : sinT[(size_t)t * half + i];
        const float a = p[0], b = p[half];
        p[0] = a * c - b * s;
        p[half] = b * c + a * s;
    }
}

// ---- attention as batched float32 matrix products on the matrix cores, one batch entry per head:
//     forward   S = scale Q K^T   (A B^T),   P = causal soft-max(S),   O = P V   (A B)
//     backward  dP = dO V^T       (A B^T),   dS = P (dP - rowsum(P dP)),
//               dQ = scale dS K   (A B),     dK = scale sum_heads dS^T Q,   dV = sum_heads P^T dO   (A^T B)
// P and dS are T x T per head with zeros above the diagonal, so the products that read them only walk the keys a block
// of rows can see, and the products that write T x T skip the blocks above the diagonal.
//
// C[b] (+)= alpha * sum over the heads of b's group of op(A)[h] op(B)[h]; a workgroup (4 waves) owns a 64 x 64 block of C,
// a wave 16 rows of it.  v_mfma_f32_16x16x4_f32: lane l supplies A(row l % 16, k) and B(k, col l % 16) for one k of its
// group l / 16; a lane takes four consecutive k per step -- one 16-byte load where k is the contiguous index of the
// operand, four loads (each contiguous across the 16 lanes of a group) where it is not.
struct FitBmm {
    const float *A, *B;
    float* C;
    int M, N, K;               // C is M x N per batch entry, K the summed index
    int lda, ldb, ldc;         // elements between consecutive rows of the stored operands
    size_t a_hs, b_hs, c_bs;   // elements between heads of A, of B; between batch entries of C
    int a_div, b_div;          // operand A / B of head h is stored at index h / a_div, h / b_div (grouped KV heads)
    int inner;                 // heads summed into one batch entry (1, or the group size for dK / dV)
    int causal;                // 0: all k.  1: A is P-like (row m sees k < block end).  2: A^T of P-like (row m sees k >= m's block)
    int skip_upper;            // C is T x T and only the blocks on and below the diagonal are wanted
    float alpha;
    int accumulate;
};
template <bool AT, bool BT>
__global__ __launch_bounds__(256) void k_fit_bmm(FitBmm p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r16 = lane & 15, gq = lane >> 4;
    const int mb = blockIdx.x * 64, n0 = blockIdx.y * 64, bz = blockIdx.z;
    if (p.skip_upper && n0 > mb + 63) return;
    const int m0 = mb + wave * 16;
    int k_lo = 0, k_hi = p.K;
    if (p.causal == 1) k_hi = min(p.K, mb + 64);
    if (p.causal == 2) k_lo = mb;
    f32x4 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int am = min(m0 + r16, p.M - 1);
    const bool va = (p.lda & 3) == 0 && (p.a_hs & 3) == 0, vb = (p.ldb & 3) == 0 && (p.b_hs & 3) == 0;   // 16-byte loads allowed
    int bn[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) bn[c] = min(n0 + c * 16 + r16, p.N - 1);
    for (int hh = 0; hh < p.inner; ++hh) {
        const int h = bz * p.inner + hh;
        const float* Ah = p.A + (size_t)(h / p.a_div) * p.a_hs;
        const float* Bh = p.B + (size_t)(h / p.b_div) * p.b_hs;
        for (int k0 = k_lo; k0 < k_hi; k0 += 16) {
            const int kb = k0 + gq * 4;                     // this lane group's four k
            float a[4], b[4][4];
            if (kb + 4 <= p.K) {
                if (!AT && va) {
                    const f32x4 t = *reinterpret_cast<const f32x4*>(Ah + (size_t)am * p.lda + kb);
                    a[0] = t.x; a[1] = t.y; a[2] = t.z; a[3] = t.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) a[e] = AT ? Ah[(size_t)(kb + e) * p.lda + am] : Ah[(size_t)am * p.lda + kb + e];
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (BT && vb) {
                        const f32x4 t = *reinterpret_cast<const f32x4*>(Bh + (size_t)bn[c] * p.ldb + kb);
                        b[c][0] = t.x; b[c][1] = t.y; b[c][2] = t.z; b[c][3] = t.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            b[c][e] = BT ? Bh[(size_t)bn[c] * p.ldb + kb + e] : Bh[(size_t)(kb + e) * p.ldb + bn[c]];
                    }
                }
            } else {   // the ragged end of the summed index: k past the end contribute zeros (read from the last valid k)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = min(kb + e, p.K - 1);
                    const float av = AT ? Ah[(size_t)k * p.lda + am] : Ah[(size_t)am * p.lda + k];
                    a[e] = kb + e < p.K ? av : 0.f;
#pragma unroll
                    for (int c = 0; c < 4; ++c) b[c][e] = BT ? Bh[(size_t)bn[c] * p.ldb + k] : Bh[(size_t)k * p.ldb + bn[c]];
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[c][e], acc[c], 0, 0, 0);
        }
    }
    float* Cb = p.C + (size_t)bz * p.c_bs;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int n = n0 + c * 16 + r16;
        const float v[4] = {acc[c].x, acc[c].y, acc[c].z, acc[c].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int m = m0 + gq * 4 + e;
            if (m < p.M && n < p.N) {
                float* o = Cb + (size_t)m * p.ldc + n;
                *o = (p.accumulate ? *o : 0.f) + p.alpha * v[e];
            }
        }
    }
}
// causal soft-max of the rows of S [H][T][T] in place: row (h, i) over j <= i, zeros past i.  One wave per row.
__global__ __launch_bounds__(64) void k_fit_softmax(float* __restrict__ S, int T) {
    float* row = S + ((size_t)blockIdx.y * T + blockIdx.x) * T;
    const int i = blockIdx.x, lane = threadIdx.x;
    float mx = -INFINITY;
    for (int j = lane; j <= i; j += 64) mx = fmaxf(mx, row[j]);
    mx = wave_max(mx);
    float l = 0.f;
    for (int j = lane; j <= i; j += 64) l += expf(row[j] - mx);
    l = fit_wave_sum(l);
    const float inv = 1.0f / l;
    for (int j = lane; j < T; j += 64) row[j] = j <= i ? expf(row[j] - mx) * inv : 0.f;
}
// dS = P (dP - sum_j P dP) over j <= i, zeros past i; dP [H][T][T] is overwritten.  One wave per row.
__global__ __launch_bounds__(64) void k_fit_softmax_bwd(const float* __restrict__ P, float* __restrict__ dP, int T) {
    const size_t o = ((size_t)blockIdx.y * T + blockIdx.x) * T;
    const int i = blockIdx.x, lane = threadIdx.x;
    float D = 0.f;
    for (int j = lane; j <= i; j += 64) D += P[o + j] * dP[o + j];
    D = fit_wave_sum(D);
    for (int j = lane; j < T; j += 64) dP[o + j] = j <= i ? P[o + j] * (dP[o + j] - D) : 0.f;
}

// ---- SwiGLU: act = silu(gate) up; backward: dgate = dact up s (1 + gate (1 - s)), dup = dact gate s, s = sigmoid(gate)
__global__ __launch_bounds__(256) void k_fit_swiglu(const float* __restrict__ gt, const float* __restrict__ up, size_t n,
                                                    float* __restrict__ act) {
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) {
        const float s = 1.0f / (1.0f + expf(-gt[e]));
        act[e] = gt[e] * s * up[e];
    }
}
__global__ __launch_bounds__(256) void k_fit_swiglu_bwd(const float* __restrict__ dact, const float* __restrict__ gt,
                                                        const float* __restrict__ up, size_t n, float* __restrict__ dgt,
                                                        float* __restrict__ dup) {
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) {
        const float g = gt[e], s = 1.0f / (1.0f + expf(-g)), da = dact[e];
        dup[e] = da * g * s;
        dgt[e] = da * up[e] * (s * (1.0f + g * (1.0f - s)));
    }
}

// ---- cross-entropy of row t against tokens[t + 1] for t < T - 1, and its gradient in place: the loss is the mean over
// the T - 1 rows, so dlogits = (softmax - onehot) / (T - 1); row T - 1 has no target and gets zeros. --------------------
__global__ __launch_bounds__(256) void k_fit_ce(float* __restrict__ z, const int* __restrict__ tokens, int T, int V, double* loss) {
    __shared__ float sh[16];
    const int t = blockIdx.x;
    float* row = z + (size_t)t * V;
    if (t == T - 1) {
        for (int c = threadIdx.x; c < V; c += blockDim.x) row[c] = 0.f;
        return;
    }
    float mx = -INFINITY;
    for (int c = threadIdx.x; c < V; c += blockDim.x) mx = fmaxf(mx, row[c]);
    mx = fit_block_max(mx, sh);
    float l = 0.f;
    for (int c = threadIdx.x; c < V; c += blockDim.x) l += expf(row[c] - mx);
    l = fit_block_sum(l, sh);
    const int tgt = tokens[t + 1];
    const float inv = 1.0f / l, w = 1.0f / (float)(T - 1);
    if (threadIdx.x == 0) atomicAdd(loss, (double)(-(row[tgt] - mx - logf(l))) * (double)w);
    __syncthreads();
    for (int c = threadIdx.x; c < V; c += blockDim.x) row[c] = (expf(row[c] - mx) * inv - (c == tgt ? 1.f : 0.f)) * w;
}

// ---- transposed copy of a bfloat16 matrix, written in the tile order of the GEMM's weight operand (pf_tile_weights):
// the copy is W^T [C][R] of src W [R][C]; its tile t = rows 16 t .. (columns of W), step s = values 32 s .. of a row (rows of
// W), lane l's 16 bytes = row l % 16 of the tile, values (l / 16) * 8 .. of the step, at l * 16 of the kilobyte
// (t * R / 32 + s).  One workgroup per 32 x 32 block of W, through LDS.  R a multiple of 32, C of 16. ------------------
__global__ __launch_bounds__(256) void k_fit_transpose(const bf16_t* __restrict__ src, int R, int C, bf16_t* __restrict__ dst) {
    __shared__ bf16_t tile[32][33];
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int y = ty; y < 32; y += 8)
        if (r0 + y < R && c0 + tx < C) tile[y][tx] = src[(size_t)(r0 + y) * C + c0 + tx];
    __syncthreads();
    if (threadIdx.x < 128) {   // unit = (column c of W, quarter gq of the step): 8 values W[r0 + gq * 8 ..][c]
        const int cl = threadIdx.x & 31, gq = threadIdx.x >> 5, c = c0 + cl;
        if (c < C) {
            unsigned w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                w[e] = (unsigned)tile[gq * 8 + 2 * e][cl] | ((unsigned)tile[gq * 8 + 2 * e + 1][cl] << 16);
            const size_t frag = (size_t)(c >> 4) * (R >> 5) + (r0 >> 5);
            *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(dst) + frag * PF_FRAG_BYTES + gq * 256 + (c & 15) * 16) =
                u32x4{w[0], w[1], w[2], w[3]};
        }
    }
}

// ---- Gram matrix G += A A^T of a float32 matrix A [T][w] on the float32 matrix cores.  A workgroup (4 waves) adds the
// contribution of one stretch of columns to a 128 x 128 block of G (G zeroed beforehand; the stretches of a block meet
// in float32 atomic adds -- storing the stretches apart and adding them later costs more than the atomics do).  v_mfma_f32_16x16x4_f32: lane l supplies A[row l % 16][k = l / 16] and B[k = l / 16][col l % 16]
// and holds D[rows 4 (l / 16) .. + 3][col l % 16]; a lane loads four consecutive k of its row at once, and which four k a
// lane group takes does not matter as long as both operands take the same.  G is symmetric: only the 128 x 128 blocks on
// and above the diagonal are computed (the others stay zero) and k_fit_dot counts a block above the diagonal twice. ----
__global__ __launch_bounds__(256) void k_fit_gram(const float* __restrict__ A, int T, int w, int k_per_wg, float* __restrict__ G) {
    if (blockIdx.y < blockIdx.x) return;   // below the diagonal
    // a workgroup owns a 128 x 128 block of G, wave (wr, wc) its 64 x 64 quarter: 4 + 4 operand loads feed 64 instructions
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r16 = lane & 15, gq = lane >> 4;
    const int i0 = blockIdx.x * 128 + (wave >> 1) * 64, j0 = blockIdx.y * 128 + (wave & 1) * 64;
    const int k_lo = blockIdx.z * k_per_wg, k_hi = min(w, k_lo + k_per_wg);
    const float *ar[4], *br[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        ar[c] = A + (size_t)min(i0 + c * 16 + r16, T - 1) * w + gq * 4;
        br[c] = A + (size_t)min(j0 + c * 16 + r16, T - 1) * w + gq * 4;
    }
    f32x4 acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int k0 = k_lo; k0 < k_hi; k0 += 16) {
        f32x4 a[4], b[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            a[c] = *reinterpret_cast<const f32x4*>(ar[c] + k0);
            b[c] = *reinterpret_cast<const f32x4*>(br[c] + k0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r].x, b[c].x, acc[r][c], 0, 0, 0);
                acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r].y, b[c].y, acc[r][c], 0, 0, 0);
                acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r].z, b[c].z, acc[r][c], 0, 0, 0);
                acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r].w, b[c].w, acc[r][c], 0, 0, 0);
            }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = j0 + c * 16 + r16;
            const float v[4] = {acc[r][c].x, acc[r][c].y, acc[r][c].z, acc[r][c].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = i0 + r * 16 + gq * 4 + e;
                if (i < T && j < T) atomicAdd(G + (size_t)i * T + j, v[e]);
            }
        }
}
// *acc += sum_{t,t'} G1[t][t'] G2[t][t'] for two symmetric T x T matrices of which only the 128 x 128 blocks on and above
// the diagonal are filled: a block above the diagonal stands for its mirror image as well
__global__ __launch_bounds__(256) void k_fit_dot(const float* __restrict__ G1, const float* __restrict__ G2, int T, double* acc) {
    __shared__ float sh[16];
    float s = 0.f;
    const size_t n = (size_t)T * T;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) {
        const int i = (int)(e / T), j = (int)(e - (size_t)i * T), bi = i >> 7, bj = j >> 7;
        if (bj >= bi) s += (bj > bi ? 2.f : 1.f) * G1[e] * G2[e];
    }
    s = fit_block_sum(s, sh);
    if (threadIdx.x == 0) atomicAdd(acc, (double)s);
}

}  // namespace sdfp
