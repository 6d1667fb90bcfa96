// One-launch forward: every phase of every layer in a single persistent kernel (one workgroup per CU),
// separated by grid-wide barriers.  Before arriving at a barrier each wave has already issued the first
// weight loads of the NEXT projection phase into its register ring: those loads depend on no activation, so
// the HBM read stream keeps flowing while the barrier, the attention phase and the activation staging run.
// This is what removes the per-kernel ramp/drain cost that bounds a launch-per-phase forward at batch 1.
#pragma once
#include "sdfp_attn.hip.h"
#include "sdfp_gemv.hip.h"

namespace sdfp {

struct LayerW {   // device-resident table entry, one per layer
    const void *wq, *wk, *wv, *wo, *wg, *wu, *wd;
    const float *attn_norm, *ffn_norm;
};

struct FwdArgs {
    const LayerW* layers;          // [n_layers]
    const unsigned char* skip;     // [n_layers] SD_SKIP_* bits, or nullptr: run every layer (the target model)
    int n_layers;
    LayerDims L;
    Rows rows;
    DevState* st;
    const int* prompt;
    const void* tok_emb;
    const float* final_norm;
    const void* lm_head;
    char* kv;
    float *h, *q, *att, *a;
    const float *cosT, *sinT;
    float *part_o, *part_ml;
    unsigned* att_counters;
    HeadOut head;
    int head_run, head_row_from;
    float eps;
    unsigned* bar;                 // BAR_WORDS counters, all left at 0 except the sticky time-out flag
    unsigned spin_limit;
    unsigned long long* trace;     // optional timeline of workgroup 0 (100 MHz ticks), or nullptr
    int trace_cap;
};

// Grid-wide barrier over co-resident workgroups, fence-free: everything exchanged across it travels through
// agent-coherent accesses, so arriving only needs this workgroup's stores to be acknowledged (the
// __syncthreads waits for them).  Two levels keep the atomic traffic short: workgroups count into one of
// BAR_GROUPS counters (own cache lines), the last arrival of a group bumps the global counter that everyone
// polls.  `epoch` = number of barriers passed so far in this launch + 1.  The wait is bounded: after
// spin_limit polls the sticky flag is raised and every later barrier falls through, so the kernel always
// terminates; the host reports the flag as SD_ETIMEOUT.
constexpr int BAR_GROUPS = 8;
constexpr int BAR_STRIDE = 16;                          // unsigneds between counters (64-byte lines)
constexpr int BAR_WORDS = BAR_STRIDE * (BAR_GROUPS + 2);
// layout: bar[0] global count, bar[BAR_STRIDE] time-out flag, bar[BAR_STRIDE * (2 + g)] group g
__device__ __forceinline__ void bar_arrive(unsigned* bar, unsigned epoch, int wg, int n_wg) {
    const int ng = n_wg < BAR_GROUPS ? n_wg : BAR_GROUPS;
    const int grp = wg % ng;
    const unsigned gsize = (unsigned)((n_wg - grp + ng - 1) / ng);
    const unsigned old = atomicAdd(bar + BAR_STRIDE * (2 + grp), 1u);
    if (old + 1 == epoch * gsize) atomicAdd(bar, 1u);
}
__device__ __forceinline__ void bar_wait(unsigned* bar, unsigned epoch, int n_wg, unsigned spin_limit) {
    const unsigned target = epoch * (unsigned)(n_wg < BAR_GROUPS ? n_wg : BAR_GROUPS);
    unsigned spins = 0;
    while (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
        if (++spins > spin_limit || (spins & 1023u) == 0) {
            if (spins > spin_limit) atomicExch(bar + BAR_STRIDE, 1u);
            if (__hip_atomic_load(bar + BAR_STRIDE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
        }
    }
}
__device__ __forceinline__ void grid_barrier(unsigned* bar, unsigned epoch, int wg, int n_wg, unsigned spin_limit) {
    __syncthreads();
    if (threadIdx.x == 0) {
        bar_arrive(bar, epoch, wg, n_wg);
        bar_wait(bar, epoch, n_wg, spin_limit);
    }
    __syncthreads();
}

enum { PH_NONE = 0, PH_QKV, PH_OPROJ, PH_GATEUP, PH_DOWN, PH_HEAD };
struct PhaseRef { int kind, layer; };

template <typename WT, int MT, int D>
struct Forward {
    const FwdArgs& A;
    float* lds;
    int wg, n_wg, M, pos0, n_trace;
    Ring<D> ring;
    HeadOp<WT, MT> head_op;

    __device__ __forceinline__ Forward(const FwdArgs& a, float* l) : A(a), lds(l) {}

    // timeline entry: (tag << 56) | ticks; tag = phase kind * 2 + {0: phase body done, 1: barrier passed}
    __device__ __forceinline__ void mark(int tag) {
        if (A.trace != nullptr && wg == 0 && threadIdx.x == 0 && n_trace < A.trace_cap)
            A.trace[n_trace++] = ((unsigned long long)tag << 56) | (wall_clock64() & 0x00FFFFFFFFFFFFFFull);
    }
    __device__ __forceinline__ void sync_all(unsigned& epoch, int kind) {
        mark(kind * 2);
        grid_barrier(A.bar, ++epoch, wg, n_wg, A.spin_limit);
        mark(kind * 2 + 1);
    }

    __device__ __forceinline__ int skip_of(int l) const { return A.skip ? A.skip[l] : 0; }

    // first projection phase at or after (layer l, sub-layer s): s = 0 attention, 1 feed-forward
    __device__ __forceinline__ PhaseRef next_from(int l, int s) const {
        for (; l < A.n_layers; ++l, s = 0) {
            const int sk = skip_of(l);
            if (s == 0 && !(sk & 1)) return PhaseRef{PH_QKV, l};
            if (!(sk & 2)) return PhaseRef{PH_GATEUP, l};
        }
        return PhaseRef{A.head_run ? PH_HEAD : PH_NONE, 0};
    }

    __device__ __forceinline__ QkvOp<WT, MT> qkv_op(int l) const {
        const LayerW& w = A.layers[l];
        const size_t plane = (size_t)A.L.Hkv * A.L.max_seq * A.L.hd;
        QkvOp<WT, MT> op;
        op.wq = (const WT*)w.wq; op.wk = (const WT*)w.wk; op.wv = (const WT*)w.wv;
        op.kc = reinterpret_cast<WT*>(A.kv) + (size_t)(2 * l) * plane;
        op.vc = op.kc + plane;
        op.q = A.q; op.cosT = A.cosT; op.sinT = A.sinT; op.L = A.L; op.M = M; op.pos0 = pos0;
        return op;
    }
    __device__ __forceinline__ ResidOp<WT, MT> oproj_op(int l) const {
        ResidOp<WT, MT> op;
        op.w = (const WT*)A.layers[l].wo; op.h = A.h; op.N = A.L.d; op.K = A.L.H * A.L.hd; op.M = M;
        return op;
    }
    __device__ __forceinline__ GateUpOp<WT, MT> gateup_op(int l) const {
        GateUpOp<WT, MT> op;
        op.wg = (const WT*)A.layers[l].wg; op.wu = (const WT*)A.layers[l].wu; op.a = A.a;
        op.F = A.L.F; op.d = A.L.d; op.M = M;
        return op;
    }
    __device__ __forceinline__ ResidOp<WT, MT> down_op(int l) const {
        ResidOp<WT, MT> op;
        op.w = (const WT*)A.layers[l].wd; op.h = A.h; op.N = A.L.d; op.K = A.L.F; op.M = M;
        return op;
    }

    template <class Op>
    __device__ __forceinline__ void prefetch_op(const Op& op) {
        GemvPhase<WT, MT, D, Op> ph;
        ph.setup(op, wg, n_wg);
        ph.prefetch(op, ring);
    }
    template <class Op>
    __device__ __forceinline__ void run_op(Op& op, const float* x, const float* gain) {
        GemvPhase<WT, MT, D, Op> ph;
        ph.setup(op, wg, n_wg);
        ph.run(op, ring, x, gain, A.eps, lds);
        stores_done();   // epilogue stores acknowledged before this wave prefetches and heads for the barrier
    }

    __device__ __forceinline__ void prefetch(PhaseRef p) {
        switch (p.kind) {
            case PH_QKV: prefetch_op(qkv_op(p.layer)); break;
            case PH_OPROJ: prefetch_op(oproj_op(p.layer)); break;
            case PH_GATEUP: prefetch_op(gateup_op(p.layer)); break;
            case PH_DOWN: prefetch_op(down_op(p.layer)); break;
            case PH_HEAD: prefetch_op(head_op); break;
            default: break;
        }
    }

    __device__ __forceinline__ void attention(int l) {
        const size_t plane = (size_t)A.L.Hkv * A.L.max_seq * A.L.hd;
        const WT* kc = reinterpret_cast<const WT*>(A.kv) + (size_t)(2 * l) * plane;
        const WT* vc = kc + plane;
        AttnArgs aa;
        aa.q = A.q; aa.att = A.att; aa.part_o = A.part_o; aa.part_ml = A.part_ml; aa.counters = A.att_counters;
        aa.L = A.L; aa.rows = A.rows; aa.st = A.st;
        const int n_active = (pos0 + M + ATT_SL - 1) / ATT_SL;
        const int n_items = n_active * A.L.Hkv;
        for (int it = wg; it < n_items; it += n_wg) {
            const int g = it / n_active, split = it - g * n_active;
            attn_dispatch<WT>(kc, vc, aa, lds, split, g);
            __syncthreads();
        }
    }

    __device__ __forceinline__ void run() {
        wg = blockIdx.x; n_wg = gridDim.x;
        M = A.rows.M;
        pos0 = row_pos(A.rows, A.st, 0);
        unsigned epoch = 0;
        n_trace = 0;
        mark(0);
        head_op.init((const WT*)A.lm_head, A.L.V, A.L.d, M - A.head_row_from, A.head.logits);

        PhaseRef nxt = next_from(0, 0);
        prefetch(nxt);
        // a1: embedding gather, spread over the whole grid
        {
            const int d = A.L.d;
            for (int idx = (wg * WG_THREADS + threadIdx.x) * 4; idx < M * d; idx += n_wg * WG_THREADS * 4) {
                const int m = idx / d, k = idx - m * d;
                const WT* e = (const WT*)A.tok_emb + (size_t)row_tok(A.rows, A.st, A.prompt, m) * d + k;
                f32x4 v = {ST<WT>::ld(e), ST<WT>::ld(e + 1), ST<WT>::ld(e + 2), ST<WT>::ld(e + 3)};
                st_coh4(A.h + idx, v);
            }
            stores_done();
        }
        sync_all(epoch, 7);

        for (int l = 0; l < A.n_layers; ++l) {
            const int sk = skip_of(l);
            const LayerW& w = A.layers[l];
            if (!(sk & 1)) {
                { auto op = qkv_op(l); run_op(op, A.h, w.attn_norm); }
                prefetch(PhaseRef{PH_OPROJ, l});
                sync_all(epoch, PH_QKV);
                attention(l);
                sync_all(epoch, 6);
                { auto op = oproj_op(l); run_op(op, A.att, nullptr); }
                prefetch(next_from(l, 1));
                sync_all(epoch, PH_OPROJ);
            }
            if (!(sk & 2)) {
                { auto op = gateup_op(l); run_op(op, A.h, w.ffn_norm); }
                prefetch(PhaseRef{PH_DOWN, l});
                sync_all(epoch, PH_GATEUP);
                { auto op = down_op(l); run_op(op, A.a, nullptr); }
                prefetch(next_from(l + 1, 0));
                sync_all(epoch, PH_DOWN);
            }
        }
        if (A.head_run) {
            run_op(head_op, A.h + (size_t)A.head_row_from * A.L.d, A.final_norm);
            head_publish(head_op, A.head, lds, wg);
        }
        // last barrier: every workgroup arrives, only workgroup 0 waits; it reduces the arg-max partials and
        // re-arms the counters for the next launch
        __syncthreads();
        ++epoch;
        if (wg != 0) {
            if (threadIdx.x == 0) bar_arrive(A.bar, epoch, wg, n_wg);
            return;
        }
        if (threadIdx.x == 0) {
            bar_arrive(A.bar, epoch, wg, n_wg);
            bar_wait(A.bar, epoch, n_wg, A.spin_limit);
        }
        __syncthreads();
        mark(PH_HEAD * 2);
        if (A.head_run) head_final(A.head, M - A.head_row_from, n_wg, A.st);
        mark(PH_HEAD * 2 + 1);
        if (A.trace != nullptr && threadIdx.x == 0) A.trace[A.trace_cap] = (unsigned long long)n_trace;
        if (threadIdx.x < BAR_GROUPS + 2 && threadIdx.x != 1) st_coh(A.bar + BAR_STRIDE * threadIdx.x, 0u);
    }
};

template <typename WT, int MT, int D>
__global__ __launch_bounds__(WG_THREADS, 1) void k_forward(FwdArgs args) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    Forward<WT, MT, D> f(args, lds);
    f.run();
}

}  // namespace sdfp
