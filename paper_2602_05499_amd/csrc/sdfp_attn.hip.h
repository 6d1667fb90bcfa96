// Causal attention of M <= 16 rows over the contiguous KV cache (step a3 of the forward).
#pragma once
#include "sdfp_common.hip.h"

namespace sdfp {

// ---- a3: causal attention of M rows over the contiguous cache, split along positions --------------------
// A workgroup handles one split of ATT_SL positions of one KV head for all rows
// and all query heads of the group -- or, where splits x KV heads leave most of the grid idle (grouped-query models:
// 8 KV heads x 9 splits for 48 query vectors each), for one of n_qparts shares of those query vectors; a query's
// arithmetic does not depend on which others share its workgroup, and the KV head's merge counter then expects
// n_qparts arrivals per split.  K and V rows are read once, straight from the cache with coalesced
// row loads (lanes split head_dim), scores are reduced on the DPP network, soft-max statistics per split go
// to the workspace, and the last workgroup of a KV head to finish merges the splits in ascending order.
struct AttnArgs {
    const float* q;    // [M][H*hd]
    float* att;        // [M][H*hd]
    float* part_o;     // [n_splits][MAX_ROWS][part_H][hd]: partials of query heads part_h0 .. part_h0 + part_H - 1
    float* part_ml;    // [n_splits][MAX_ROWS][part_H][2]
    int part_H, part_h0;   // the forward kernel keeps all heads (H, 0); the prompt path one KV head's group per region
    unsigned* counters;  // merge counters, left at 0: of KV head g at counters[g] (forward kernels), or the caller's own (panel)
    LayerDims L;
    Rows rows;
    const DevState* st;
};

constexpr int ATT_PPW = ATT_SL / NWAVE;   // positions per wave per split (16)

// LDS: scores [ATT_QC][ATT_SL] + per-wave output partials [NWAVE][ATT_QC][hd] + (max, sum) [ATT_QC][2] + the
// query vectors of the group [M * H / Hkv][hd]
// (qc = query vectors per pass: ATT_QC in the forward kernels, ATT_QC_PANEL in the prompt path's kernel, which wants
// two workgroups on a compute unit -- its chains of dependent LDS and cross-lane operations hide one another only
// with more waves)
constexpr int ATT_QC_PANEL = 8;
// floats of the per-wave output partials; the prompt path's kernel keeps the four quarter sums of every score there
// first ([4][qc][ATT_SL]; see attn_split, PANEL), and stages no queries
__host__ __device__ constexpr size_t attn_ored_floats(int hd, int qc, bool panel) {
    return panel && 4 * ATT_SL > NWAVE * hd ? (size_t)4 * qc * ATT_SL : (size_t)NWAVE * qc * hd;
}
__host__ __device__ constexpr size_t attn_lds_bytes(int hd, int nq, int qc = ATT_QC, bool panel = false) {
    return sizeof(float) * (size_t)(qc * ATT_SL + attn_ored_floats(hd, qc, panel) + 2 * qc + (panel ? 0 : nq * hd));
}

// four consecutive dims of a cache row, kept in storage form.  Plain loads: within one launch a cache line of
// this layer's planes, or of the query buffer, is first read after the barrier that follows its last write.
template <typename WT> struct Row4;
template <> struct Row4<bf16_t> {
    u32x2 r;
    __device__ __forceinline__ void zero() { r = u32x2{0u, 0u}; }
    __device__ __forceinline__ void load(const bf16_t* p) {
        r = ld_act8(p);
    }
    __device__ __forceinline__ void get(float (&f)[4]) const {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xFFFF0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xFFFF0000u);
    }
};
template <> struct Row4<float> {
    f32x4 r;
    __device__ __forceinline__ void zero() { r = f32x4{0.f, 0.f, 0.f, 0.f}; }
    __device__ __forceinline__ void load(const float* p) { r = ld_act4(p); }
    __device__ __forceinline__ void get(float (&f)[4]) const { f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w; }
};

// LPP = lanes per position = hd / 4 (each lane holds 4 consecutive dims of a K or V row)
// MROWS: the number of rows of the launch when known at compile time, else 0
// PANEL (prompt path): one workgroup runs the splits of a (16-row chunk, KV head) one after another, split 0 first, into
// partial buffers of its own that hold one KV head's group.  Same arithmetic, operation for operation; what differs
// is how the work lies on the lanes and what surrounds it: the scores are computed with a key per lane and the queries
// in scalar registers (below; no cross-lane steps, no staging of the queries), the last call merges (no counter: every
// partial is the workgroup's own, one wait for the stores in front of the merge), and values are widened once instead
// of once per query (there are registers for it here).  (Skipping the row loads whose positions all lie beyond the
// chunk's last row was tried: the branches cost more than the work they save.)  false (forward kernels): all heads,
// one counter per KV head; these kernels have no register to spare for any of that.
// LONGCTX: the context can hold more than 8 splits (max_seq > 8 * ATT_SL): more than 8 splits are merged by merge_long
// (statistics staged in LDS, partials in batches).  The forward kernels of contexts that cannot hold as many keep the
// compact one-split-at-a-time loop for that case instead (never run there): they sit at the register limit, and
// merge_long's scalar registers alone cost their forwards 1 %.
template <typename WT, int LPP, int MROWS, bool PANEL = false, bool LONGCTX = true>
__device__ __forceinline__ void attn_split(const WT* __restrict__ kc, const WT* __restrict__ vc, const AttnArgs& a,
                                           float* lds, int split, int g, int qpart = 0, int n_qparts = 1) {
    const int part_H = PANEL ? a.part_H : a.L.H, part_h0 = PANEL ? a.part_h0 : 0;
    unsigned* const counter = PANEL ? a.counters : a.counters + g;
    constexpr int QC = PANEL ? ATT_QC_PANEL : ATT_QC;   // query vectors per pass
    constexpr int PPL = 64 / LPP;            // positions covered by one wave-wide row load
    constexpr int NL = ATT_PPW / PPL > 0 ? ATT_PPW / PPL : 1;   // row loads per wave per split
    static_assert(NL * PPL * NWAVE == ATT_SL || PPL > ATT_PPW, "split length must tile");
    const int hd = a.L.hd, H = a.L.H, Hkv = a.L.Hkv, grp = H / Hkv, M = MROWS > 0 ? MROWS : a.rows.M;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pos0 = row_pos(a.rows, a.st, 0);
    const int Ltot = pos0 + M;
    const int n_active = (Ltot + ATT_SL - 1) / ATT_SL;
    const int start = split * ATT_SL, npos = min(ATT_SL, Ltot - start);
    float* sc = lds;                               // [QC][ATT_SL]
    float* ored = sc + QC * ATT_SL;            // [NWAVE][QC][hd]  (PANEL: first the quarter sums [4][QC][ATT_SL])
    float* mls = ored + attn_ored_floats(hd, QC, PANEL);   // [QC][2]
    const float scale = 1.0f / sqrtf((float)hd);
    const int sub = lane / LPP, dl = (lane % LPP) * 4;   // position slot inside a row load, first dim of the lane

    // positions owned by this wave: j = (l * NWAVE + wave) * PPL + sub  (interleaved over waves)
    // K and V stay in their storage form in registers (bf16: 2 registers per 4 dims) and are widened on use
    Row4<WT> kr4[PANEL ? 1 : NL], vr4[NL];
#pragma unroll
    for (int l = 0; l < NL; ++l) {
        const int j = (l * NWAVE + wave) * PPL + sub;
        if (!PANEL) kr4[PANEL ? 0 : l].zero();
        vr4[l].zero();
        if (j < npos) {
            if (!PANEL) kr4[PANEL ? 0 : l].load(kc + ((size_t)g * a.L.max_seq + start + j) * hd + dl);
            vr4[l].load(vc + ((size_t)g * a.L.max_seq + start + j) * hd + dl);
        }
    }
    // PANEL, scores: a key per lane.  Wave w takes quarter w % 4 of head_dim for the 64 positions (w / 4) * 64 + lane, so
    // that the queries come from scalar registers (a wave's lanes all multiply by the same query values) and nothing
    // crosses lanes: per query and key a quarter costs hd / 4 multiply-adds and the adds of its part of the tree, where
    // the layout above (a key across hd / 4 lanes) spends as much again on the cross-lane steps of every 4 dims.
    constexpr int DG = PANEL ? LPP / 4 : 1;   // 4-dim groups per quarter
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int kq_r = wave_u & 3, kq_j = (wave_u >> 2) * 64 + lane;
    float kq[DG][4];
    if constexpr (PANEL) {
        static_assert(!PANEL || (LPP % 4 == 0 && ATT_SL == 128 && NWAVE == 8), "four quarters x two halves of a split");
#pragma unroll
        for (int dg = 0; dg < DG; ++dg) {
            Row4<WT> t;
            t.zero();
            if (kq_j < npos) t.load(kc + ((size_t)g * a.L.max_seq + start + kq_j) * hd + (kq_r * DG + dg) * 4);
            t.get(kq[dg]);
        }
    }
    const int nq = M * grp;   // query vectors: qi = m * grp + gi
    // every query vector of the group goes to LDS now, behind the K / V loads: one memory round trip for all
    float* qs = mls + 2 * QC;   // [nq][hd]
    for (int e0 = tid * 4; e0 < nq * hd && !PANEL; e0 += 4 * WG_THREADS * 4) {
        f32x4 qv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * WG_THREADS * 4;
            if (e < nq * hd) {
                const int qi = e / hd, dim = e - qi * hd, m = qi / grp, hq = g * grp + (qi - m * grp);
                qv[u] = ld_act4(a.q + (size_t)m * H * hd + (size_t)hq * hd + dim);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * WG_THREADS * 4;
            if (e < nq * hd) *reinterpret_cast<f32x4*>(qs + e) = qv[u];
        }
    }
    __syncthreads();
    // PANEL: the rows widened once
    float vw[PANEL ? NL : 1][4];
    if constexpr (PANEL) {
#pragma unroll
        for (int l = 0; l < NL; ++l) vr4[l].get(vw[l]);
    }
    // this call's share of the query vectors (all of them unless the caller dealt a split to several workgroups)
    const int q_from = (nq * qpart) / n_qparts, q_to = (nq * (qpart + 1)) / n_qparts;
    for (int q0 = q_from; q0 < q_to; q0 += QC) {
        const int nqc = min(QC, q_to - q0);
        // scores: the lane group of a position reduces its 4-dim partial dot products on the DPP network
        for (int ql = 0; ql < nqc && !PANEL; ++ql) {
            const int qi = q0 + ql, m = qi / grp;
            const f32x4 qv = *reinterpret_cast<const f32x4*>(qs + (size_t)qi * hd + dl);
#pragma unroll
            for (int l = 0; l < NL; ++l) {
                const int j = (l * NWAVE + wave) * PPL + sub;
                float kf[4];
                kr4[PANEL ? 0 : l].get(kf);
                float s = kf[0] * qv.x;
                s = fmaf(kf[1], qv.y, s); s = fmaf(kf[2], qv.z, s); s = fmaf(kf[3], qv.w, s);
                s = group_sum_dpp<LPP>(s);
                if ((lane % LPP) == LPP - 1 && j < ATT_SL)
                    sc[ql * ATT_SL + j] = (j < npos && start + j <= pos0 + m) ? s * scale : -INFINITY;
            }
        }
        // PANEL: the same sums in the same order -- per 4 dims a product and three fused multiply-adds, then the tree of
        // group_sum_dpp, which adds neighbours, pairs of neighbours and so on: this wave's quarter of it here (the tree
        // over the quarter's 4-dim groups), the two levels above it, (Q0 + Q1) + (Q2 + Q3), where the scores are read
        for (int ql = 0; ql < nqc && PANEL; ++ql) {
            const int qi = q0 + ql, m = qi / grp, hq = g * grp + (qi - m * grp);
            const SDFP_CONST float* qrow = as_const(a.q) + (size_t)m * H * hd + (size_t)hq * hd + kq_r * (DG * 4);   // wave-uniform
            float t[DG];
#pragma unroll
            for (int dg = 0; dg < DG; ++dg) {
                float p = kq[dg][0] * qrow[dg * 4];
                p = fmaf(kq[dg][1], qrow[dg * 4 + 1], p); p = fmaf(kq[dg][2], qrow[dg * 4 + 2], p);
                t[dg] = fmaf(kq[dg][3], qrow[dg * 4 + 3], p);
            }
#pragma unroll
            for (int w = 1; w < DG; w <<= 1)
#pragma unroll
                for (int i = 0; i + w < DG; i += 2 * w) t[i] = add_rn(t[i], t[i + w]);
            ored[(kq_r * QC + ql) * ATT_SL + kq_j] = t[0];
        }
        __syncthreads();
        // soft-max statistics per query (one wave per query); probabilities written back in place
        for (int ql = wave; ql < nqc; ql += NWAVE) {
            float s0, s1;
            if constexpr (PANEL) {
                const int m = (q0 + ql) / grp;
                auto score = [&](int j) {
                    const float* qsum = ored + ql * ATT_SL + j;
                    const float sum = add_rn(add_rn(qsum[0], qsum[QC * ATT_SL]), add_rn(qsum[2 * QC * ATT_SL], qsum[3 * QC * ATT_SL]));
                    return (j < npos && start + j <= pos0 + m) ? sum * scale : -INFINITY;
                };
                s0 = score(lane); s1 = score(64 + lane);
            } else {
                s0 = sc[ql * ATT_SL + lane]; s1 = sc[ql * ATT_SL + 64 + lane];
            }
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
                float vf[4];
                if constexpr (PANEL) { vf[0] = vw[l][0]; vf[1] = vw[l][1]; vf[2] = vw[l][2]; vf[3] = vw[l][3]; }
                else vr4[l].get(vf);
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = fmaf(p, vf[e], o[e]);
            }
            // fold the PPL position slots of the wave (lanes with equal lane % LPP) in a fixed order
#pragma unroll
            for (int off = LPP; off < 64; off <<= 1)
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] += __shfl_xor(o[e], off);
            if (sub == 0)
                *reinterpret_cast<f32x4*>(ored + ((size_t)wave * QC + ql) * hd + dl) = f32x4{o[0], o[1], o[2], o[3]};
        }
        __syncthreads();
        for (int idx = tid; idx < nqc * hd; idx += WG_THREADS) {
            const int ql = idx / hd, dim = idx - ql * hd;
            float o = 0.f;
#pragma unroll
            for (int w = 0; w < NWAVE; ++w) o += ored[((size_t)w * QC + ql) * hd + dim];
            const int qi = q0 + ql, m = qi / grp, hq = g * grp + (qi - m * grp);
            st_coh(a.part_o + (((size_t)split * MAX_ROWS + m) * part_H + hq - part_h0) * hd + dim, o);
            if (dim == 0) {
                float* ml = a.part_ml + (((size_t)split * MAX_ROWS + m) * part_H + hq - part_h0) * 2;
                st_coh(ml, mls[ql * 2]); st_coh(ml + 1, mls[ql * 2 + 1]);
            }
        }
        __syncthreads();
    }
    // last workgroup of this KV head merges the splits
    if constexpr (PANEL) {
        if (split != n_active - 1) return;   // uniform; the partials are this workgroup's own, the last call merges
        stores_done();
        __syncthreads();
    } else {
        stores_done();
        __syncthreads();
        __shared__ unsigned s_last;
        if (tid == 0) s_last = (atomic_inc_g(counter) == (unsigned)(n_active * n_qparts - 1)) ? 1u : 0u;
        __syncthreads();
        if (!s_last) return;
    }
    // One output: the splits' partials weighted by exp(max_s - max) in ascending split order.
    auto merge = [&](int idx) {
        const int qi = idx / hd, dim = idx - qi * hd, m = qi / grp, hq = g * grp + (qi - m * grp);
        const int hp = hq - part_h0;   // head index inside the partial buffers
        float num = 0.f, den = 0.f;
        if (LONGCTX || n_active <= 8) {   // every statistic and partial of this output in flight at once
            float ms[8], ls[8], os[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                ms[s] = -INFINITY; ls[s] = 0.f; os[s] = 0.f;
                if (s < n_active) {
                    const float* ml = a.part_ml + (((size_t)s * MAX_ROWS + m) * part_H + hp) * 2;
                    ms[s] = ld_coh(ml); ls[s] = ld_coh(ml + 1);
                    os[s] = ld_coh(a.part_o + (((size_t)s * MAX_ROWS + m) * part_H + hp) * hd + dim);
                }
            }
            float gmax = -INFINITY;
#pragma unroll
            for (int s = 0; s < 8; ++s) gmax = fmaxf(gmax, ms[s]);
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                if (s < n_active) {
                    const float w = (ms[s] > -INFINITY) ? __expf(ms[s] - gmax) : 0.f;
                    num = fmaf(w, os[s], num);
                    den = fmaf(w, ls[s], den);
                }
            }
        } else {   // more splits, one at a time: compact, and slow (the LONGCTX instances never come here, see merge_long)
            float gmax = -INFINITY;
            for (int s = 0; s < n_active; ++s)
                gmax = fmaxf(gmax, ld_coh(a.part_ml + (((size_t)s * MAX_ROWS + m) * part_H + hp) * 2));
            for (int s = 0; s < n_active; ++s) {
                const float* ml = a.part_ml + (((size_t)s * MAX_ROWS + m) * part_H + hp) * 2;
                const float ms = ld_coh(ml), ls = ld_coh(ml + 1);
                const float w = (ms > -INFINITY) ? __expf(ms - gmax) : 0.f;
                const float o = ld_coh(a.part_o + (((size_t)s * MAX_ROWS + m) * part_H + hp) * hd + dim);
                num = fmaf(w, o, num);
                den = fmaf(w, ls, den);
            }
        }
        st_coh(a.att + (size_t)m * H * hd + (size_t)hq * hd + dim, num / den);
    };
    // More splits (contexts beyond 1024 positions): the same operations per output in the same order.  The statistics
    // of a chunk of query vectors go to LDS first (the scores and output partials there are dead by now; one round
    // trip for all of them), so that an output's only loads are its partials, MB splits in flight at a time.  (One
    // split at a time, statistics included, is a chain of some 70 memory round trips per output at 33 splits: 120 us
    // per layer of a five-row forward with 20 query vectors per KV head at 4096 positions, most of that layer's time.)
    auto merge_long = [&](int q_lo, int q_hi) {
        const int cap = QC * ATT_SL + NWAVE * QC * hd;                // floats of the scores and the output partials
        constexpr int MB = 8;
        float* stat = lds;                                            // [queries of the chunk][n_active][2]
        const int qb = max(1, cap / (2 * n_active));
        for (int qc0 = q_lo; qc0 < q_hi; qc0 += qb) {
            const int nqc = min(qb, q_hi - qc0);
            __syncthreads();   // the previous chunk (or whatever used this LDS before) has been read
            for (int e = tid; e < nqc * n_active; e += WG_THREADS) {
                const int ql = e / n_active, sp = e - ql * n_active, qi = qc0 + ql;
                const int m = qi / grp, hp = g * grp + (qi - m * grp) - part_h0;
                const u32x2 v = ld_coh8(a.part_ml + (((size_t)sp * MAX_ROWS + m) * part_H + hp) * 2);
                stat[e * 2] = __uint_as_float(v.x); stat[e * 2 + 1] = __uint_as_float(v.y);
            }
            __syncthreads();
            // A thread takes W consecutive outputs of a query vector: one partial load per split, the weights once.  One
            // row: W = 1, which covers the group's query vectors with an output per thread (the one-row kernels have no
            // registers for more: 16-byte partials put three of theirs into scratch memory and cost 4 us per layer).
            constexpr int W = MROWS == 1 ? 1 : 4;
            const int per_q = W == 4 ? LPP : hd;
            for (int u = tid; u < nqc * per_q; u += WG_THREADS) {
                const int ql = u / per_q, d0 = (u - ql * per_q) * W, qi = qc0 + ql;
                const int m = qi / grp, hq = g * grp + (qi - m * grp), hp = hq - part_h0;
                const float* sq = stat + (size_t)ql * n_active * 2;
                float gmax = -INFINITY;
                for (int sp = 0; sp < n_active; ++sp) gmax = fmaxf(gmax, sq[sp * 2]);
                const float* o0 = a.part_o + ((size_t)m * part_H + hp) * hd + d0;
                const size_t o_split = (size_t)MAX_ROWS * part_H * hd;
                float num[W], den = 0.f;
#pragma unroll
                for (int e = 0; e < W; ++e) num[e] = 0.f;
                for (int s0 = 0; s0 < n_active; s0 += MB) {
                    float os[MB][W];
#pragma unroll
                    for (int sp = 0; sp < MB; ++sp) {
#pragma unroll
                        for (int e = 0; e < W; ++e) os[sp][e] = 0.f;
                        if (s0 + sp < n_active) {
                            const float* src = o0 + (size_t)(s0 + sp) * o_split;
                            if constexpr (W == 4) {
                                const f32x4 v = ld_coh4(src);
                                os[sp][0] = v.x; os[sp][1] = v.y; os[sp][2] = v.z; os[sp][3] = v.w;
                            } else {
                                os[sp][0] = ld_coh(src);
                            }
                        }
                    }
#pragma unroll
                    for (int sp = 0; sp < MB; ++sp) {
                        if (s0 + sp < n_active) {
                            const float ms = sq[(s0 + sp) * 2], ls = sq[(s0 + sp) * 2 + 1];
                            const float w = (ms > -INFINITY) ? __expf(ms - gmax) : 0.f;
#pragma unroll
                            for (int e = 0; e < W; ++e) num[e] = fmaf(w, os[sp][e], num[e]);
                            den = fmaf(w, ls, den);
                        }
                    }
                }
                float* dst = a.att + (size_t)m * H * hd + (size_t)hq * hd + d0;
                if constexpr (W == 4) st_coh4(dst, f32x4{num[0] / den, num[1] / den, num[2] / den, num[3] / den});
                else st_coh(dst, num[0] / den);
            }
        }
    };
    auto merge_queries = [&](int q_lo, int q_hi) {   // query vectors [q_lo, q_hi) of the group
        if (LONGCTX && n_active > 8) {
            merge_long(q_lo, q_hi);
        } else {
            for (int idx = q_lo * hd + tid; idx < q_hi * hd; idx += WG_THREADS) merge(idx);
        }
    };
    if (MROWS >= 2) {
        // The rows go to the next phase without a grid barrier, and its readers poll row 0 only: rows 1.. first,
        // their acknowledgement by every wave, row 0 last.  Row 0 is the first grp query vectors.
        merge_queries(grp, nq);
        stores_done();
        __syncthreads();
        merge_queries(0, grp);
    } else {
        merge_queries(0, nq);
    }
    if constexpr (!PANEL) {
        stores_done();
        if (tid == 0) st_coh(counter, 0u);   // re-arm (coherent: the next arrivals come from other XCDs)
    }
}

// head_dim -> lanes per position of the attention kernel (one kernel instance per head_dim keeps the code small)
__host__ __device__ constexpr int attn_lpp(int hd) { return hd / 4; }

}  // namespace sdfp
