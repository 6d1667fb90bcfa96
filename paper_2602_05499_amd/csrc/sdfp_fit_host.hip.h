// Host side of the FIT layer scores (Eq. 11; Alg. 1 Stage A): workspace layout, the forward that keeps what the backward
// needs, the backward, and the squared gradient norms per sub-layer (kernels and the method in sdfp_fit.hip.h).
// Included at the end of sdfp_api.hip: the kernels it shares with the prompt path are defined once, in that unit.
#pragma once
#include "sdfp_fit.hip.h"
#include "sdfp.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

using namespace sdfp;

namespace {

inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct FitDims {
    int L, d, H, Hkv, hd, F, V, T;
    int hq, hkv;
};
bool fit_dims(const sd_config* c, int T, FitDims& D) {
    if (!c || c->dtype != SD_BF16) return false;
    if (c->n_layers < 1 || c->n_heads < 1 || c->n_kv_heads < 1 || c->n_heads % c->n_kv_heads) return false;
    if (c->head_dim < 16 || c->head_dim > 128 || (c->head_dim & (c->head_dim - 1))) return false;
    if (T < 2 || T > FIT_MAX_T) return false;
    D = FitDims{c->n_layers, c->d_model, c->n_heads, c->n_kv_heads, c->head_dim, c->d_ffn, c->vocab, T,
                c->n_heads * c->head_dim, c->n_kv_heads * c->head_dim};
    // every width is a reduction length of some product: whole 64-byte steps of bfloat16, and whole 16-row tiles
    for (int wdt : {D.d, D.hq, D.hkv, D.F, D.V})
        if (wdt < 32 || wdt % 32) return false;
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return false;
    return true;
}

// byte offsets into the workspace
struct FitCarve {
    size_t tokens, cosT, sinT, scores, x1, rs1, rs2, rsf, qr, kr, v, P, att, x2, gt, up;   // kept by the forward
    size_t n, act, xs, logits, wT, dh, dn, dq, dk, dv, datt, dact, dgt, dup, dS, GX, GD, shares;   // temporaries
    size_t total;
};
FitCarve fit_carve(const FitDims& D) {
    FitCarve k;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = up256(off + bytes); return o; };
    const size_t T = D.T, L = D.L, f = sizeof(float);
    const size_t wmax = (size_t)std::max({D.d, D.hq, D.F, D.V});
    k.tokens = take(T * 4);
    k.cosT = take(T * (D.hd / 2) * f); k.sinT = take(T * (D.hd / 2) * f);
    k.scores = take((2 * L + 1) * sizeof(double));
    k.x1 = take((L + 1) * T * D.d * f);
    k.rs1 = take(L * T * f); k.rs2 = take(L * T * f); k.rsf = take(T * f);
    k.qr = take(L * T * D.hq * f); k.kr = take(L * T * D.hkv * f); k.v = take(L * T * D.hkv * f);
    k.P = take(L * (size_t)D.H * T * T * f);
    k.att = take(L * T * D.hq * f); k.x2 = take(L * T * D.d * f);
    k.gt = take(L * T * D.F * f); k.up = take(L * T * D.F * f);
    k.n = take(T * D.d * f); k.act = take(T * D.F * f);
    k.xs = take(3 * pf_xs_piece(D.T, (int)wmax) * 2);
    k.logits = take(T * (size_t)D.V * f);
    k.wT = take(std::max({(size_t)D.F * D.d, (size_t)D.V * D.d, (size_t)D.hq * D.d}) * 2);
    k.dh = take(T * D.d * f); k.dn = take(T * D.d * f);
    k.dq = take(T * D.hq * f); k.dk = take(T * D.hkv * f); k.dv = take(T * D.hkv * f);
    k.datt = take(T * D.hq * f);
    k.dact = take(T * D.F * f); k.dgt = take(T * D.F * f); k.dup = take(T * D.F * f);
    k.dS = take((size_t)D.H * T * T * f);
    k.GX = take(T * T * f); k.GD = take(T * T * f);
    k.shares = take(PF_NSHARE * T * (size_t)std::max(D.d, D.hq) * f);   // per-share partial sums of a narrow product
    k.total = off;
    return k;
}

struct Fit {
    FitDims D;
    FitCarve cv;
    char* ws;
    hipStream_t st;
    int n_cu;
    char* tcache;      // room behind the workspace proper for a transposed copy of every matrix, or nullptr
    char* fcache;      // room behind that for a copy of every matrix in tile order (forward products), or nullptr
    bool tfill;        // the copies are being made (first sample of a call)
    float* f(size_t off) const { return reinterpret_cast<float*>(ws + off); }
};
// bytes of all transposed matrices (seven per layer and the output head), and where matrix `slot` of layer l sits
// (slot 0..6 = wq wk wv wo w_gate w_up w_down; layer L, slot 0 = the output head)
size_t fit_tcache_offset(const FitDims& D, int l, int slot) {
    const size_t sz[7] = {(size_t)D.hq * D.d, (size_t)D.hkv * D.d, (size_t)D.hkv * D.d, (size_t)D.d * D.hq,
                          (size_t)D.F * D.d, (size_t)D.F * D.d, (size_t)D.d * D.F};
    size_t per_layer = 0, before = 0;
    for (int i = 0; i < 7; ++i) { if (i < slot) before += up256(sz[i] * 2); per_layer += up256(sz[i] * 2); }
    return (size_t)l * per_layer + before;
}
size_t fit_tcache_bytes(const FitDims& D) { return fit_tcache_offset(D, D.L, 0) + up256((size_t)D.V * D.d * 2); }

// out (+)= X W^T: X [T][K] float32, W [N][K] bfloat16 row-major, out [T][ldo]
template <int NT, bool PARTIAL>
void fit_gemm_launch(const Fit& F, const PfGemm& a) {
    static bool attr_done = false;   // per kernel instance
    if (!attr_done) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_pf_gemm<PF_PLAIN, NT, PARTIAL>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, PF_LDS_BYTES);
        attr_done = true;
    }
    const unsigned grid = (unsigned)((a.n_nt * a.n_groups + 7) / 8 * 8 * a.my);
    hipLaunchKernelGGL((k_pf_gemm<PF_PLAIN, NT, PARTIAL>), dim3(grid), dim3(WG_THREADS), PF_LDS_BYTES, F.st, a);
}
// A weight operand: the matrix and whether it lies in tile order (pf_tile_weights) or row-major
struct FitW { const void* p; bool tiled; };
void fit_gemm(const Fit& F, FitW Wt, int N, int K, const float* X, float* out, int ldo, bool accumulate) {
    const void* W = Wt.p;
    const int T = F.D.T;
    bf16_t* xs = reinterpret_cast<bf16_t*>(F.ws + F.cv.xs);
    hipLaunchKernelGGL(k_pf_split, dim3(1024), dim3(256), 0, F.st, X, (const float*)nullptr, T, K, xs, pf_xs_piece(T, K));
    PfGemm a;
    std::memset(&a, 0, sizeof(a));
    a.w[0] = reinterpret_cast<const bf16_t*>(W);
    a.wt = Wt.tiled ? a.w[0] : nullptr;
    a.xs = xs; a.xs_piece = pf_xs_piece(T, K); a.Kd = K; a.n_tiles = N / 16; a.M = T;
    a.out = out; a.ldo = ldo; a.accumulate = accumulate ? 1 : 0;
    a.my = (T + PF_TM - 1) / PF_TM; a.n_groups = 1;
    const int fill = (F.n_cu * 3) / 8;
    if (((a.n_tiles + 23) / 24) * a.my >= fill) {
        a.n_nt = (a.n_tiles + 23) / 24;
        fit_gemm_launch<3, false>(F, a);
    } else if (N <= std::max(F.D.d, F.D.hq) && ((a.n_tiles + 31) / 32) * a.my * PF_NSHARE >= fill) {
        // few outputs but many rows: large tiles, a tile's shares dealt to several workgroups (as the prompt path does
        // for its O and down projections), the shares' sums added in order by k_pf_residual
        a.n_nt = (a.n_tiles + 31) / 32;
        while (a.n_groups < PF_NSHARE && a.n_nt * a.my * a.n_groups < (F.n_cu * 3) / 4) a.n_groups *= 2;
        a.part = F.f(F.cv.shares); a.part_arr = (size_t)T * N; a.part_ld = N;
        fit_gemm_launch<4, true>(F, a);
        if (!accumulate) (void)hipMemsetAsync(out, 0, (size_t)T * N * 4, F.st);
        hipLaunchKernelGGL(k_pf_residual, dim3(512), dim3(256), 0, F.st, out, F.f(F.cv.shares), a.part_arr, T * N / 4);
    } else {
        a.n_nt = (a.n_tiles + 7) / 8;
        fit_gemm_launch<1, false>(F, a);
    }
}
// W^T of W [R][C], in tile order, into the scratch matrix, or into (from the second sample on: out of) the call's cache
FitW fit_transposed(const Fit& F, const void* W, int R, int C, int l, int slot) {
    bf16_t* dst = reinterpret_cast<bf16_t*>(F.tcache ? F.tcache + fit_tcache_offset(F.D, l, slot) : F.ws + F.cv.wT);
    if (!F.tcache || F.tfill)
        hipLaunchKernelGGL(k_fit_transpose, dim3((C + 31) / 32, (R + 31) / 32), dim3(256), 0, F.st,
                           reinterpret_cast<const bf16_t*>(W), R, C, dst);
    return FitW{dst, true};
}
// W [N][K] for a forward product: the caller's row-major matrix, or its copy in tile order when the call has a cache
FitW fit_forward(const Fit& F, const void* W, int N, int K, int l, int slot) {
    if (!F.fcache) return FitW{W, false};
    bf16_t* dst = reinterpret_cast<bf16_t*>(F.fcache + fit_tcache_offset(F.D, l, slot));
    if (F.tfill) {
        PfGemm a;
        std::memset(&a, 0, sizeof(a));
        a.w[0] = reinterpret_cast<const bf16_t*>(W); a.Kd = K; a.n_tiles = N / 16;
        hipLaunchKernelGGL(k_pf_tile_weights<PF_PLAIN>, dim3(2048), dim3(256), 0, F.st, a, dst);
    }
    return FitW{dst, true};
}
void fit_gram(const Fit& F, const float* A, int w, float* G) {
    const int T = F.D.T, tb = (T + 127) / 128;
    (void)hipMemsetAsync(G, 0, (size_t)T * T * 4, F.st);
    int ks = std::max(1, std::min(FIT_GRAM_SLICES, w / 128));
    const int k_per = ((w + ks - 1) / ks + 15) / 16 * 16;
    ks = (w + k_per - 1) / k_per;
    hipLaunchKernelGGL(k_fit_gram, dim3(tb, tb, ks), dim3(256), 0, F.st, A, T, w, k_per, G);
}
// *acc += || dY^T X ||_F^2 with the Gram matrix of X already in GX
void fit_weight_norm(const Fit& F, const float* dY, int w_out, double* acc) {
    float* GD = F.f(F.cv.GD);
    fit_gram(F, dY, w_out, GD);
    hipLaunchKernelGGL(k_fit_dot, dim3(256), dim3(256), 0, F.st, F.f(F.cv.GX), GD, F.D.T, acc);
}

template <bool AT, bool BT>
void fit_bmm(const Fit& F, const FitBmm& p, int batch) {
    hipLaunchKernelGGL((k_fit_bmm<AT, BT>), dim3((p.M + 63) / 64, (p.N + 63) / 64, batch), dim3(256), 0, F.st, p);
}
// attention forward of all heads: P = softmax(scale q k^T) into P [H][T][T], att = P v
void fit_attention_fwd(const Fit& F, const float* q, const float* k, const float* v, float* P, float* att) {
    const FitDims& D = F.D;
    const int T = D.T, grp = D.H / D.Hkv;
    FitBmm s;
    std::memset(&s, 0, sizeof(s));
    s.A = q; s.B = k; s.C = P; s.M = T; s.N = T; s.K = D.hd; s.lda = D.hq; s.ldb = D.hkv; s.ldc = T;
    s.a_hs = D.hd; s.b_hs = D.hd; s.c_bs = (size_t)T * T; s.a_div = 1; s.b_div = grp; s.inner = 1;
    s.skip_upper = 1; s.alpha = 1.0f / std::sqrt((float)D.hd);
    fit_bmm<false, true>(F, s, D.H);
    hipLaunchKernelGGL(k_fit_softmax, dim3(T, D.H), dim3(64), 0, F.st, P, T);
    FitBmm o;
    std::memset(&o, 0, sizeof(o));
    o.A = P; o.B = v; o.C = att; o.M = T; o.N = D.hd; o.K = T; o.lda = T; o.ldb = D.hkv; o.ldc = D.hq;
    o.a_hs = (size_t)T * T; o.b_hs = D.hd; o.c_bs = D.hd; o.a_div = 1; o.b_div = grp; o.inner = 1;
    o.causal = 1; o.alpha = 1.0f;
    fit_bmm<false, false>(F, o, D.H);
}
// attention backward: datt [T][hq] -> dq [T][hq], dk, dv [T][hkv]; dS [H][T][T] is scratch
void fit_attention_bwd(const Fit& F, const float* datt, const float* q, const float* k, const float* v, const float* P,
                       float* dS, float* dq, float* dk, float* dv) {
    const FitDims& D = F.D;
    const int T = D.T, grp = D.H / D.Hkv;
    const float scale = 1.0f / std::sqrt((float)D.hd);
    FitBmm a;
    std::memset(&a, 0, sizeof(a));                       // dP = dO v^T
    a.A = datt; a.B = v; a.C = dS; a.M = T; a.N = T; a.K = D.hd; a.lda = D.hq; a.ldb = D.hkv; a.ldc = T;
    a.a_hs = D.hd; a.b_hs = D.hd; a.c_bs = (size_t)T * T; a.a_div = 1; a.b_div = grp; a.inner = 1;
    a.skip_upper = 1; a.alpha = 1.0f;
    fit_bmm<false, true>(F, a, D.H);
    hipLaunchKernelGGL(k_fit_softmax_bwd, dim3(T, D.H), dim3(64), 0, F.st, P, dS, T);
    FitBmm b;
    std::memset(&b, 0, sizeof(b));                       // dq = scale dS k
    b.A = dS; b.B = k; b.C = dq; b.M = T; b.N = D.hd; b.K = T; b.lda = T; b.ldb = D.hkv; b.ldc = D.hq;
    b.a_hs = (size_t)T * T; b.b_hs = D.hd; b.c_bs = D.hd; b.a_div = 1; b.b_div = grp; b.inner = 1;
    b.causal = 1; b.alpha = scale;
    fit_bmm<false, false>(F, b, D.H);
    FitBmm c;
    std::memset(&c, 0, sizeof(c));                       // dk = scale sum_heads dS^T q
    c.A = dS; c.B = q; c.C = dk; c.M = T; c.N = D.hd; c.K = T; c.lda = T; c.ldb = D.hq; c.ldc = D.hkv;
    c.a_hs = (size_t)T * T; c.b_hs = D.hd; c.c_bs = D.hd; c.a_div = 1; c.b_div = 1; c.inner = grp;
    c.causal = 2; c.alpha = scale;
    fit_bmm<true, false>(F, c, D.Hkv);
    c.A = P; c.B = datt; c.C = dv; c.alpha = 1.0f;       // dv = sum_heads P^T dO
    fit_bmm<true, false>(F, c, D.Hkv);
}

// one sample: forward, loss, backward, scores[0..L) += attention sub-layers, scores[L..2L) += feed-forward sub-layers,
// scores[2L] = loss of this sample
void fit_sample(const Fit& F, const sd_config* cfg, const sd_weights* w) {
    const FitDims& D = F.D;
    const FitCarve& cv = F.cv;
    const int T = D.T, L = D.L;
    const size_t Td = (size_t)T * D.d, Tq = (size_t)T * D.hq, Tk = (size_t)T * D.hkv, TF = (size_t)T * D.F;
    const size_t PP = (size_t)D.H * T * T;
    const int* tokens = reinterpret_cast<const int*>(F.ws + cv.tokens);
    const float *cosT = F.f(cv.cosT), *sinT = F.f(cv.sinT);
    double* scores = reinterpret_cast<double*>(F.ws + cv.scores);
    float *n = F.f(cv.n), *act = F.f(cv.act);
    auto ew_grid = [](size_t cnt) { return dim3((unsigned)std::min<size_t>(2048, (cnt + 255) / 256)); };

    // ---- forward
    hipLaunchKernelGGL(k_pf_embed, dim3(T), dim3(256), 0, F.st, tokens, reinterpret_cast<const bf16_t*>(w->tok_emb), D.d,
                       D.V, F.f(cv.x1));
    for (int l = 0; l < L; ++l) {
        float *x1 = F.f(cv.x1) + l * Td, *x1n = F.f(cv.x1) + (l + 1) * Td, *x2 = F.f(cv.x2) + l * Td;
        float *qr = F.f(cv.qr) + l * Tq, *kr = F.f(cv.kr) + l * Tk, *v = F.f(cv.v) + l * Tk, *att = F.f(cv.att) + l * Tq;
        float *gt = F.f(cv.gt) + l * TF, *up = F.f(cv.up) + l * TF;
        hipLaunchKernelGGL(k_fit_rmsnorm, dim3(T), dim3(256), 0, F.st, x1, (const float*)w->attn_norm[l], D.d, cfg->rms_eps, n,
                           F.f(cv.rs1) + (size_t)l * T);
        fit_gemm(F, fit_forward(F, w->wq[l], D.hq, D.d, l, 0), D.hq, D.d, n, qr, D.hq, false);
        fit_gemm(F, fit_forward(F, w->wk[l], D.hkv, D.d, l, 1), D.hkv, D.d, n, kr, D.hkv, false);
        fit_gemm(F, fit_forward(F, w->wv[l], D.hkv, D.d, l, 2), D.hkv, D.d, n, v, D.hkv, false);
        hipLaunchKernelGGL(k_fit_rope, dim3(T), dim3(256), 0, F.st, qr, D.H, D.hd, cosT, sinT, 0);
        hipLaunchKernelGGL(k_fit_rope, dim3(T), dim3(256), 0, F.st, kr, D.Hkv, D.hd, cosT, sinT, 0);
        fit_attention_fwd(F, qr, kr, v, F.f(cv.P) + l * PP, att);
        (void)hipMemcpyAsync(x2, x1, Td * 4, hipMemcpyDeviceToDevice, F.st);
        fit_gemm(F, fit_forward(F, w->wo[l], D.d, D.hq, l, 3), D.d, D.hq, att, x2, D.d, true);
        hipLaunchKernelGGL(k_fit_rmsnorm, dim3(T), dim3(256), 0, F.st, x2, (const float*)w->ffn_norm[l], D.d, cfg->rms_eps, n,
                           F.f(cv.rs2) + (size_t)l * T);
        fit_gemm(F, fit_forward(F, w->w_gate[l], D.F, D.d, l, 4), D.F, D.d, n, gt, D.F, false);
        fit_gemm(F, fit_forward(F, w->w_up[l], D.F, D.d, l, 5), D.F, D.d, n, up, D.F, false);
        hipLaunchKernelGGL(k_fit_swiglu, ew_grid(TF), dim3(256), 0, F.st, gt, up, TF, act);
        (void)hipMemcpyAsync(x1n, x2, Td * 4, hipMemcpyDeviceToDevice, F.st);
        fit_gemm(F, fit_forward(F, w->w_down[l], D.d, D.F, l, 6), D.d, D.F, act, x1n, D.d, true);
    }
    float* hL = F.f(cv.x1) + (size_t)L * Td;
    float* logits = F.f(cv.logits);
    hipLaunchKernelGGL(k_fit_rmsnorm, dim3(T), dim3(256), 0, F.st, hL, (const float*)w->final_norm, D.d, cfg->rms_eps, n,
                       F.f(cv.rsf));
    fit_gemm(F, fit_forward(F, w->lm_head, D.V, D.d, L, 0), D.V, D.d, n, logits, D.V, false);
    (void)hipMemsetAsync(scores + 2 * L, 0, sizeof(double), F.st);
    hipLaunchKernelGGL(k_fit_ce, dim3(T), dim3(256), 0, F.st, logits, tokens, T, D.V, scores + 2 * L);

    // ---- backward.  dh: gradient of the residual stream entering the part of the network still to be walked.
    float *dh = F.f(cv.dh), *dn = F.f(cv.dn), *dq = F.f(cv.dq), *dk = F.f(cv.dk), *dv = F.f(cv.dv), *datt = F.f(cv.datt);
    float *dact = F.f(cv.dact), *dgt = F.f(cv.dgt), *dup = F.f(cv.dup), *dS = F.f(cv.dS), *GX = F.f(cv.GX);
    fit_gemm(F, fit_transposed(F, w->lm_head, D.V, D.d, L, 0), D.d, D.V, logits, dn, D.d, false);
    hipLaunchKernelGGL(k_fit_rmsnorm_bwd, dim3(T), dim3(256), 0, F.st, hL, (const float*)w->final_norm, F.f(cv.rsf), dn, D.d,
                       (const float*)nullptr, dh);
    for (int l = L - 1; l >= 0; --l) {
        float *x1 = F.f(cv.x1) + l * Td, *x2 = F.f(cv.x2) + l * Td;
        float *qr = F.f(cv.qr) + l * Tq, *kr = F.f(cv.kr) + l * Tk, *v = F.f(cv.v) + l * Tk, *att = F.f(cv.att) + l * Tq;
        float *gt = F.f(cv.gt) + l * TF, *up = F.f(cv.up) + l * TF, *P = F.f(cv.P) + l * PP;
        const float *rs1 = F.f(cv.rs1) + (size_t)l * T, *rs2 = F.f(cv.rs2) + (size_t)l * T;
        double *s_attn = scores + l, *s_ffn = scores + L + l;
        // feed-forward sub-layer: h_out = x2 + act W_down^T
        hipLaunchKernelGGL(k_fit_swiglu, ew_grid(TF), dim3(256), 0, F.st, gt, up, TF, act);
        fit_gram(F, act, D.F, GX);
        fit_weight_norm(F, dh, D.d, s_ffn);                                              // w_down
        fit_gemm(F, fit_transposed(F, w->w_down[l], D.d, D.F, l, 6), D.F, D.d, dh, dact, D.F, false);
        hipLaunchKernelGGL(k_fit_swiglu_bwd, ew_grid(TF), dim3(256), 0, F.st, dact, gt, up, TF, dgt, dup);
        hipLaunchKernelGGL(k_fit_rmsnorm, dim3(T), dim3(256), 0, F.st, x2, (const float*)w->ffn_norm[l], D.d, cfg->rms_eps, n, dn);
        // (the reciprocal RMS written to dn above is scratch: rs2 is the kept one)
        fit_gram(F, n, D.d, GX);
        fit_weight_norm(F, dgt, D.F, s_ffn);                                             // w_gate
        fit_weight_norm(F, dup, D.F, s_ffn);                                             // w_up
        fit_gemm(F, fit_transposed(F, w->w_gate[l], D.F, D.d, l, 4), D.d, D.F, dgt, dn, D.d, false);
        fit_gemm(F, fit_transposed(F, w->w_up[l], D.F, D.d, l, 5), D.d, D.F, dup, dn, D.d, true);
        hipLaunchKernelGGL(k_fit_dgain_sumsq, dim3((D.d + 63) / 64), dim3(1024), 0, F.st, x2, rs2, dn, T, D.d, s_ffn);   // ffn_norm
        hipLaunchKernelGGL(k_fit_rmsnorm_bwd, dim3(T), dim3(256), 0, F.st, x2, (const float*)w->ffn_norm[l], rs2, dn, D.d,
                           (const float*)dh, dh);                                        // dh = gradient at x2
        // attention sub-layer: x2 = x1 + att W_o^T
        fit_gram(F, att, D.hq, GX);
        fit_weight_norm(F, dh, D.d, s_attn);                                             // wo
        fit_gemm(F, fit_transposed(F, w->wo[l], D.d, D.hq, l, 3), D.hq, D.d, dh, datt, D.hq, false);
        fit_attention_bwd(F, datt, qr, kr, v, P, dS, dq, dk, dv);
        hipLaunchKernelGGL(k_fit_rope, dim3(T), dim3(256), 0, F.st, dq, D.H, D.hd, cosT, sinT, 1);
        hipLaunchKernelGGL(k_fit_rope, dim3(T), dim3(256), 0, F.st, dk, D.Hkv, D.hd, cosT, sinT, 1);
        hipLaunchKernelGGL(k_fit_rmsnorm, dim3(T), dim3(256), 0, F.st, x1, (const float*)w->attn_norm[l], D.d, cfg->rms_eps, n, dn);
        fit_gram(F, n, D.d, GX);
        fit_weight_norm(F, dq, D.hq, s_attn);                                            // wq
        fit_weight_norm(F, dk, D.hkv, s_attn);                                           // wk
        fit_weight_norm(F, dv, D.hkv, s_attn);                                           // wv
        fit_gemm(F, fit_transposed(F, w->wq[l], D.hq, D.d, l, 0), D.d, D.hq, dq, dn, D.d, false);
        fit_gemm(F, fit_transposed(F, w->wk[l], D.hkv, D.d, l, 1), D.d, D.hkv, dk, dn, D.d, true);
        fit_gemm(F, fit_transposed(F, w->wv[l], D.hkv, D.d, l, 2), D.d, D.hkv, dv, dn, D.d, true);
        hipLaunchKernelGGL(k_fit_dgain_sumsq, dim3((D.d + 63) / 64), dim3(1024), 0, F.st, x1, rs1, dn, T, D.d, s_attn);  // attn_norm
        hipLaunchKernelGGL(k_fit_rmsnorm_bwd, dim3(T), dim3(256), 0, F.st, x1, (const float*)w->attn_norm[l], rs1, dn, D.d,
                           (const float*)dh, dh);                                        // dh = gradient at x1
    }
}

}  // namespace

extern "C" {

size_t sd_fit_workspace_bytes(const sd_config* cfg, int32_t T) {
    FitDims D;
    if (!fit_dims(cfg, T, D)) return 0;
    return fit_carve(D).total;
}

int sd_fit_scores(const sd_config* cfg, const sd_weights* w, const int32_t* tokens_host, int32_t n_samples, int32_t T,
                  void* ws_buf, size_t ws_bytes, void* hip_stream, double* t_attn_host, double* t_ffn_host,
                  double* loss_host) {
    FitDims D;
    if (!fit_dims(cfg, T, D) || !w || !tokens_host || n_samples < 1 || !t_attn_host || !t_ffn_host) return SD_EINVAL;
    if (!ws_buf || ((uintptr_t)ws_buf & 255)) return SD_EINVAL;
    if (!w->tok_emb || !w->lm_head || !w->final_norm) return SD_EINVAL;
    for (int l = 0; l < D.L; ++l) {
        const void* ps[9] = {w->attn_norm[l], w->wq[l], w->wk[l], w->wv[l], w->wo[l],
                             w->ffn_norm[l], w->w_gate[l], w->w_up[l], w->w_down[l]};
        for (const void* p : ps)
            if (!p || ((uintptr_t)p & 15)) return SD_EINVAL;
    }
    for (size_t i = 0; i < (size_t)n_samples * T; ++i)
        if (tokens_host[i] < 0 || tokens_host[i] >= D.V) return SD_EINVAL;
    Fit F;
    F.D = D; F.cv = fit_carve(D); F.ws = (char*)ws_buf; F.st = (hipStream_t)hip_stream;
    if (ws_bytes < F.cv.total) return SD_ENOMEM;
    // a workspace with room to spare keeps the transposed matrices from the first sample for the others
    const size_t cache = fit_tcache_bytes(D);
    F.tcache = (n_samples > 1 && ws_bytes >= F.cv.total + cache) ? F.ws + F.cv.total : nullptr;
    // ... and with room for as much again, copies in tile order for the forward products
    F.fcache = (F.tcache && ws_bytes >= F.cv.total + 2 * cache) ? F.tcache + cache : nullptr;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return SD_EHIP;
    F.n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    const int half = D.hd / 2;
    std::vector<float> cs((size_t)T * half), sn((size_t)T * half);
    for (int p = 0; p < T; ++p)
        for (int i = 0; i < half; ++i) {
            const double ang = (double)p * std::pow((double)cfg->rope_theta, -2.0 * (double)i / (double)D.hd);
            cs[(size_t)p * half + i] = (float)std::cos(ang);
            sn[(size_t)p * half + i] = (float)std::sin(ang);
        }
    if (hipMemcpyAsync(F.ws + F.cv.cosT, cs.data(), cs.size() * 4, hipMemcpyHostToDevice, F.st) != hipSuccess) return SD_EHIP;
    if (hipMemcpyAsync(F.ws + F.cv.sinT, sn.data(), sn.size() * 4, hipMemcpyHostToDevice, F.st) != hipSuccess) return SD_EHIP;
    if (hipMemsetAsync(F.ws + F.cv.scores, 0, (2 * D.L + 1) * sizeof(double), F.st) != hipSuccess) return SD_EHIP;
    std::vector<double> sc(2 * D.L + 1);
    for (int i = 0; i < n_samples; ++i) {
        if (hipMemcpyAsync(F.ws + F.cv.tokens, tokens_host + (size_t)i * T, (size_t)T * 4, hipMemcpyHostToDevice, F.st) !=
            hipSuccess)
            return SD_EHIP;
        F.tfill = i == 0;
        fit_sample(F, cfg, w);
        if (hipGetLastError() != hipSuccess) return SD_EHIP;
        if (loss_host) {   // also orders the next sample's token copy behind this sample's kernels
            if (hipMemcpyAsync(sc.data() + 2 * D.L, F.ws + F.cv.scores + 2 * D.L * sizeof(double), sizeof(double),
                               hipMemcpyDeviceToHost, F.st) != hipSuccess)
                return SD_EHIP;
            if (hipStreamSynchronize(F.st) != hipSuccess) return SD_EHIP;
            loss_host[i] = sc[2 * D.L];
        }
    }
    if (hipMemcpyAsync(sc.data(), F.ws + F.cv.scores, 2 * D.L * sizeof(double), hipMemcpyDeviceToHost, F.st) != hipSuccess)
        return SD_EHIP;
    if (hipStreamSynchronize(F.st) != hipSuccess) return SD_EHIP;
    for (int l = 0; l < D.L; ++l) {
        t_attn_host[l] = sc[l] / n_samples;
        t_ffn_host[l] = sc[D.L + l] / n_samples;
    }
    return SD_OK;
}

int sd_fit_prune_mask(const double* t_attn, const double* t_ffn, int32_t n_layers, double ratio, uint8_t* mask_out) {
    if (!t_attn || !t_ffn || !mask_out || n_layers < 1 || !(ratio >= 0.0) || !(ratio <= 1.0)) return SD_EINVAL;
    std::vector<int> order(n_layers);
    for (int l = 0; l < n_layers; ++l) order[l] = l;
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return t_attn[a] + t_ffn[a] < t_attn[b] + t_ffn[b]; });
    const int n = (int)std::floor(ratio * n_layers + 1e-12);
    std::memset(mask_out, 0, (size_t)n_layers);
    for (int i = 0; i < n; ++i) mask_out[order[i]] = (uint8_t)(SD_SKIP_ATTN | SD_SKIP_FFN);
    return SD_OK;
}


int sd_fit_prune_sublayers(const double* t_attn, const double* t_ffn, int32_t n_layers, double ratio_attn, double ratio_ffn,
                           uint8_t* mask_out) {
    if (!t_attn || !t_ffn || !mask_out || n_layers < 1) return SD_EINVAL;
    if (!(ratio_attn >= 0.0) || !(ratio_attn <= 1.0) || !(ratio_ffn >= 0.0) || !(ratio_ffn <= 1.0)) return SD_EINVAL;
    std::memset(mask_out, 0, (size_t)n_layers);
    std::vector<int> order(n_layers);
    const double* scores[2] = {t_attn, t_ffn};
    const double ratios[2] = {ratio_attn, ratio_ffn};
    const uint8_t bits[2] = {SD_SKIP_ATTN, SD_SKIP_FFN};
    for (int k = 0; k < 2; ++k) {
        for (int l = 0; l < n_layers; ++l) order[l] = l;
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return scores[k][a] < scores[k][b]; });
        const int n = (int)std::floor(ratios[k] * n_layers + 1e-12);
        for (int i = 0; i < n; ++i) mask_out[order[i]] |= bits[k];
    }
    return SD_OK;
}

}  // extern "C"
