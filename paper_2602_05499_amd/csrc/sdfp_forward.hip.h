// One-launch forward: every phase of every layer in a single persistent kernel (one workgroup per CU).  The
// phase list comes from the host (the draft model's list simply lacks the skipped sub-layers).  The weight loads
// of each wave run one turn (a ring of 16 or 8 loads) ahead of its matrix-core work and cross phase boundaries,
// so a phase starts with its first turn of weights already in registers and ends with the next phase's first
// turn on its way (the ramp-up and the tail of a phase are hidden; the boundary itself -- epilogue, hand-over of
// the rows, staging -- is not).
//
// Hand-over of rows between workgroups inside the launch.  Every activation buffer is written once per launch,
// with agent-scope stores.  Prompt chunks separate all phases by grid barriers.  The other forwards use a grid
// barrier after the embedding, before attention and at the end, and hand the rows over by the data itself
// everywhere else (see Forward::POLL and Projection).  Behind a grid barrier no address is read before it is
// written in the same launch (and the caches start every launch invalidated), so plain loads cannot hit a stale
// cache line there; a row that is polled is read with agent-scope loads, because a cached copy of it may
// predate its last store.  Buffers that ARE reused inside a launch (barrier counters, attention split partials,
// arg-max partials) are read with agent-scope loads as well.  No cache-wide write-back or invalidate is needed
// inside the kernel.
#pragma once
#include "sdfp_attn.hip.h"
#include "sdfp_stream.hip.h"

namespace sdfp {

struct FwdArgs {
    const Phase* prog;             // phase list, terminated by PK_END
    LayerDims L;
    Rows rows;
    DevState* st;
    const int* prompt;
    const void* tok_emb;
    const float *cosT, *sinT;
    float *part_o, *part_ml;
    unsigned* att_counters;
    HeadOut head;
    int head_run, head_row_from;
    int kind_units[8], kind_Kd[8]; // distribution units and reduction length of every projection kind (equal in all layers)
    float eps;
    unsigned* bar;                 // BAR_WORDS counters, all left at 0 except the sticky time-out flag
    unsigned spin_limit;
    int n_prog;                    // entries of the phase list, PK_END included
    unsigned long long* trace;     // optional timeline of workgroup 0 (100 MHz ticks), or nullptr
    int trace_cap;
    GuardRanges guard;             // used by the guard build only
};

// Grid-wide barrier over co-resident workgroups, fence-free: everything exchanged across it travels through
// agent-scope stores, so arriving only needs this workgroup's stores to be acknowledged.  Two levels keep the
// atomic traffic short: workgroups count into one of BAR_GROUPS counters (own cache lines), the last arrival
// of a group bumps the global counter that everyone polls.  `epoch` = number of barriers passed so far in
// this launch + 1.  The wait is bounded: after spin_limit polls the sticky flag is raised and every later
// barrier falls through, so the kernel always terminates; the host reports the flag as SD_ETIMEOUT.
__device__ __forceinline__ void bar_arrive(unsigned* bar, unsigned epoch, int wg, int n_wg) {
    const int ng = n_wg < BAR_GROUPS ? n_wg : BAR_GROUPS;
    const int grp = wg % ng;
    const unsigned gsize = (unsigned)((n_wg - grp + ng - 1) / ng);
    const unsigned old = atomic_inc_g(bar + BAR_STRIDE * (2 + grp));
    if (old + 1 == epoch * gsize) atomic_inc_g(bar);
}
__device__ __forceinline__ void bar_wait(unsigned* bar, unsigned epoch, int n_wg, unsigned spin_limit) {
    const unsigned target = epoch * (unsigned)(n_wg < BAR_GROUPS ? n_wg : BAR_GROUPS);
    unsigned spins = 0;
    while ((unsigned)ld_coh(reinterpret_cast<const int*>(bar)) < target) {
        if (++spins > spin_limit || (spins & 1023u) == 0) {
            if (spins > spin_limit) st_coh(bar + BAR_STRIDE, 1u);
            if (ld_coh(reinterpret_cast<const int*>(bar + BAR_STRIDE)) != 0) break;
        }
    }
}

template <typename WT, int ROLE, int LPP, int MROWS, bool SPAN, bool LONGCTX>
struct Forward {
    static constexpr int ROWS = MROWS;   // rows of the launch when known at compile time, else 0 (see Projection)
    static_assert((ROLE == 0 && MROWS == 0) || ((ROLE == 1 || ROLE == 3) && MROWS == 1) || (ROLE == 2 && MROWS >= 2),
                  "prompt chunks have any number of rows, draft and plain decode one, verify K + 1");
    // ring depth: prompt chunks stage their 16 rows in activation tiles of one or two blocks, so a shallow ring
    // (turns of two blocks) wastes fewer slots there; everywhere else the deep ring streams a little faster
    static constexpr int RD = ROLE == 0 ? 8 : RING_MAX;
    // Between two phases, rows travel either across a grid barrier or -- draft, verify and plain decode, wherever
    // the reader is a projection -- by the data itself: the reader polls row 0, which was armed at the start
    // of the launch, until every value is written (writers store row 0 last; see Projection).  That takes the
    // store acknowledgement, the counter round trips of the barrier and the skew between workgroups out of the
    // chain between a phase's last store and the next phase's first matrix-core step.  What still needs a grid barrier: embedding -> first phase (the arming must
    // be complete before anybody polls), QKV -> attention (new cache rows are not armed; the split-merge
    // counters and partial buffers are reused layer after layer) and the end of the launch.  Every activation
    // buffer of a launch is written once, so no reader can be overtaken by a later writer.
    static constexpr bool POLL = ROLE != 0;
    // The service wave's loader stops at every phase end where the wave has to wait for stores: everywhere with
    // grid barriers only (prompt chunks) and with several rows (row 0 is stored after the other rows'
    // acknowledgement); in the one-row forwards only where a grid barrier follows.
    static constexpr int HOLD = (POLL && MROWS == 1) ? 2 : 1;
    const FwdArgs& A;
    char* lds;
    int wg, n_wg, wave, M, pos0, n_trace;
    bool wt_on = false;   // wave timeline build: inside the traced window of phases
    unsigned epoch;

    __device__ __forceinline__ Forward(const FwdArgs& a, char* l) : A(a), lds(l) {}

    // timeline entry of workgroup 0's service wave: (tag << 56) | ticks; tag = phase kind * 2 + {0: phase body
    // done, 1: barrier passed}
    __device__ __forceinline__ void mark(int tag) {
#ifdef SDFP_WAVETRACE
        if (wt_on && wg == SDFP_WT_WG && (threadIdx.x & 63) == 0 && n_trace < A.trace_cap / NWAVE)
            as_global(A.trace)[wave * (A.trace_cap / NWAVE) + n_trace++] =
                ((unsigned long long)tag << 56) | (wall_clock64() & 0x00FFFFFFFFFFFFFFull);
        return;
#endif
        if (A.trace != nullptr && wg == 0 && threadIdx.x == SERVICE_WAVE * 64 && n_trace < A.trace_cap &&
            SDFP_OK(A.trace + n_trace, 8, 40))
            as_global(A.trace)[n_trace++] = ((unsigned long long)tag << 56) | (wall_clock64() & 0x00FFFFFFFFFFFFFFull);
    }
    // End of a phase.  all_stored: every wave wrote results (embedding, attention), so every wave waits for its
    // stores before the workgroup arrives.  Otherwise (projections) only the service wave stored: it alone waits
    // for the acknowledgements -- its ring is empty by then -- while the other waves go straight to the
    // workgroup barrier with their prefetched weight loads still in flight.
    __device__ __forceinline__ void sync_all(int kind, bool all_stored) {
        const bool service = wave == SERVICE_WAVE;
        if (all_stored) {
            stores_done();
            __syncthreads();
        }
        ++epoch;
        if (service) {
            if (!all_stored) stores_done();
            mark(kind * 2);
            if ((threadIdx.x & 63) == 0) {
                bar_arrive(A.bar, epoch, wg, n_wg);
                bar_wait(A.bar, epoch, n_wg, A.spin_limit);
            }
        }
        __syncthreads();
        mark(kind * 2 + 1);
    }

    __device__ __forceinline__ void embed(const Phase& p) {
        const int d = A.L.d;
        for (int idx = (wg * WG_THREADS + threadIdx.x) * 4; idx < M * d; idx += n_wg * WG_THREADS * 4) {
            const int m = idx / d, k = idx - m * d;
            // the token id comes from device state: clamp it, so that a garbage arg-max of an invalid forward (all
            // logits NaN, a timed-out barrier) cannot turn into an address outside the embedding table
            const int tok = min(max(row_tok(A.rows, A.st, A.prompt, m), 0), A.L.V - 1);
            const WT* e = (const WT*)A.tok_emb + (size_t)tok * d + k;
#ifdef SDFP_PROBE
            const f32x4 v = {0.f, 0.f, 0.f, (float)(e != nullptr)};
#else
            const f32x4 v = {ST<WT>::ld(e), ST<WT>::ld(e + 1), ST<WT>::ld(e + 2), ST<WT>::ld(e + 3)};
#endif
            st_coh4(p.out + idx, v);
        }
        if constexpr (POLL) {   // arm the rows that are handed over by data: workgroup w takes phases w + 1, w + 1 + n_wg, ...
            const unsigned a = HANDOVER_ARMED;
            const f32x4 armed = {__uint_as_float(a), __uint_as_float(a), __uint_as_float(a), __uint_as_float(a)};
            for (int ph = 1 + wg; ph < A.n_prog; ph += n_wg) {
                const SDFP_CONST Phase* q = as_const(A.prog) + ph;
                const int k = q->kind;
                if (k != PK_ATTN && k != PK_OPROJ && k != PK_GATEUP && k != PK_DOWN) continue;
#ifdef SDFP_NO_ATTN
                if (k == PK_ATTN) continue;   // timing build without attention: nobody will write these rows
#endif
                float* out = q->out;
                const int n = q->N;   // row 0 only: the row that readers poll; a multiple of 16
                for (int i = threadIdx.x * 4; i < n; i += WG_THREADS * 4) st_coh4(out + i, armed);
            }
        }
    }

    __device__ __forceinline__ void attention(const Phase& p) {
        AttnArgs aa;
        aa.q = p.xin; aa.att = p.out; aa.part_o = A.part_o; aa.part_ml = A.part_ml; aa.counters = A.att_counters;
        aa.part_H = A.L.H; aa.part_h0 = 0;
        aa.L = A.L; aa.rows = A.rows; aa.st = A.st;
        const int n_active = (pos0 + M + ATT_SL - 1) / ATT_SL;
        const int n_items = n_active * A.L.Hkv;
        // Fewer items than half the grid (grouped-query models at moderate contexts): the query vectors of an item are
        // dealt to several workgroups.  (Doing the same for the few items beyond whole rounds of the grid -- 264 items on
        // 256 workgroups -- measured the same per step: what the five-row forward gained, the one-row forwards lost.)
        const int nq = M * (A.L.H / A.L.Hkv);
        const int n_qparts = 2 * n_items <= n_wg ? min(nq, n_wg / n_items) : 1;
        for (int u = wg; u < n_items * n_qparts; u += n_wg) {
            const int it = u / n_qparts, qpart = u - it * n_qparts;
            const int g = it / n_active, split = it - g * n_active;
            attn_split<WT, LPP, ROWS, false, LONGCTX>((const WT*)p.kc, (const WT*)p.vc, aa, reinterpret_cast<float*>(lds), split, g,
                                                      qpart, n_qparts);
            __syncthreads();
        }
    }

    __device__ __forceinline__ void run() {
#ifdef SDFP_GUARD
        if (threadIdx.x == 0) s_guard = A.guard;
        __syncthreads();
#endif
        SDFP_BEACON(1);
        wg = blockIdx.x; n_wg = gridDim.x;
        wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        // The second wave of every SIMD (waves 4-7) loses the arbitration for issue slots to the first, falls
        // 2-3 us behind it in every long phase, and the workgroup waits: give it the higher priority.  (Measured:
        // one-row forwards 1.5 % faster, the five-row forward 0.7 % slower, so only the former do it.)
        if (MROWS == 1 && wave >= 4) __builtin_amdgcn_s_setprio(1);
        M = ROWS > 0 ? ROWS : A.rows.M;
        pos0 = row_pos(A.rows, A.st, 0);
        epoch = 0;
        n_trace = 0;
        mark(0);

        // this workgroup's geometry of every projection kind, kept in LDS for the whole launch
        if (threadIdx.x < LDS_ZERO_BYTES / 4) reinterpret_cast<float*>(lds + LDS_ZERO_OFF)[threadIdx.x] = 0.f;
        if (threadIdx.x < 8) {
            Geom* gt = reinterpret_cast<Geom*>(lds + LDS_GEOM_OFF) + threadIdx.x;
            const int k = threadIdx.x;
            if (is_projection(k)) *gt = make_geom<WT>(k, A.kind_units[k], A.kind_Kd[k], phase_rows(k, M, A.head_row_from), wg, n_wg);
        }
        __syncthreads();
        SDFP_BEACON(2);
        Loader<WT, RD, SPAN> ld;
        ld.init(A.prog, lds, A.L, A.head_run, wave, wave == SERVICE_WAVE ? HOLD : 0);
        SDFP_BEACON(3);
        Ring<RD> ring;
        {
            const Turn t0 = ld.next_turn();
#pragma unroll
            for (int j = 0; j < RD; ++j) ring.r[j] = ld.load(t0, j);
        }
        SDFP_BEACON(4);

        for (int ph = 0;; ++ph) {
            Phase p = load_phase(A.prog, ph);
            SDFP_BEACON(1000 + ph * 10 + p.kind);
#ifdef SDFP_WAVETRACE
            wt_on = A.trace != nullptr && ph >= SDFP_WT_LO && ph < SDFP_WT_HI;
            mark(18);
#endif
            if (p.kind == PK_END || (p.kind == PK_HEAD && !A.head_run)) break;
            const bool all_stored = p.kind == PK_EMBED || p.kind == PK_ATTN;
            if (p.kind == PK_EMBED) {
                embed(p);
            } else if (p.kind == PK_ATTN) {
#ifndef SDFP_NO_ATTN
                attention(p);
#endif
            } else {
                const int Mp = phase_rows(p.kind, M, A.head_row_from);
                if (p.kind == PK_HEAD) p.xin += (size_t)A.head_row_from * p.Kd;
                const Geom g = load_geom(lds, p.kind);   // make_geom(p.kind, p.n_units, p.Kd, Mp, wg, n_wg), computed at the start
#ifdef SDFP_WAVETRACE
                if (g.nt > 12345) mark(25);
                mark(22);
#endif
                // the first phase after the embedding reads rows that crossed a grid barrier (and were never armed);
                // coherent loads and a poll that succeeds at once are right for them too
                Projection<WT, ROWS, RD, POLL, SPAN> pj(p, A.L, lds, g, wave, pos0, A.eps, A.cosT, A.sinT, A.head,
#ifdef SDFP_WAVETRACE
                                   wt_on && wg == SDFP_WT_WG ? A.trace : nullptr,
#else
                                   A.trace,
#endif
                                   &n_trace, A.trace_cap, A.bar, A.spin_limit);
                if (p.kind == PK_HEAD && g.nt <= 0 && wave == SERVICE_WAVE && (threadIdx.x & 63) < Mp) {   // no tile here: neutral partial
                    st_coh(A.head.part_val + (size_t)wg * MAX_ROWS + (threadIdx.x & 63), -INFINITY);
                    st_coh(A.head.part_idx + (size_t)wg * MAX_ROWS + (threadIdx.x & 63), 0x7FFFFFFF);
                }
                pj.run(ring, ld, ph);
            }
            SDFP_BEACON(100000 + ph * 10 + p.kind);
            const int nk = as_const(A.prog)[ph + 1].kind;
            if (nk == PK_END || (nk == PK_HEAD && !A.head_run)) break;
            if (POLL && p.kind != PK_EMBED && is_projection(nk)) {
                // hand-over by data: only this workgroup's own waves meet (the epilogue has read its LDS inputs).
                // After attention every wave first waits for its own stores: the reset of a split-merge counter
                // must have landed long before the next layer's grid barrier lets anybody count on it again.
                mark(p.kind * 2);
                if (all_stored) stores_done();
                __syncthreads();
                mark(p.kind * 2 + 1);
            } else {
                sync_all(p.kind, all_stored);
            }
            SDFP_BEACON(200000 + ph * 10 + p.kind);
        }
        SDFP_BEACON(300000);
        // last barrier: every workgroup arrives, only workgroup 0 waits; it reduces the arg-max partials and
        // re-arms the counters for the next launch (nobody else polls them any more)
        stores_done();
        __syncthreads();
        ++epoch;
        if (threadIdx.x == SERVICE_WAVE * 64) bar_arrive(A.bar, epoch, wg, n_wg);
        if (wg != 0) { SDFP_BEACON(350000); return; }
        if (threadIdx.x == SERVICE_WAVE * 64) bar_wait(A.bar, epoch, n_wg, A.spin_limit);
        __syncthreads();
        mark(15 * 2);
        if (A.head_run) head_final(A.head, M - A.head_row_from, n_wg, A.st);
        mark(15 * 2 + 1);
        if (A.trace != nullptr && threadIdx.x == SERVICE_WAVE * 64 && SDFP_OK(A.trace + A.trace_cap, 8, 41))
            as_global(A.trace)[A.trace_cap] = (unsigned long long)n_trace;
        if (threadIdx.x < BAR_GROUPS + 2 && threadIdx.x != 1) st_coh(A.bar + BAR_STRIDE * threadIdx.x, 0u);
        SDFP_BEACON(400000);
    }
};

// One kernel instance per use of the forward (ROLE: 0 prompt rows, 1 draft row, 2 verify rows -- one instance per
// row count K + 1 --, 3 one-row plain decode) and per head_dim (LPP = head_dim / 4): each instance carries one
// attention variant and only the staging variant its row count needs.  Small code and, above all, register
// allocation without spills matter here (measured: with all attention and staging variants in one kernel the
// instance was 45 % larger, spilled 58 VGPRs to scratch and every forward was 4-8 % slower).  The ROLE also gives
// each use its own symbol in a profile.  SPAN: ring turns may go on into the next tile (see Turn); a second set of
// instances for the shapes whose weight rows do not fill whole turns (e.g. d = 5120: five blocks).  LONGCTX: contexts
// of more than 8 attention splits (max_seq > 1024) are possible, the merge of many splits is compiled in (see
// attn_split); a third doubling of the decode instances, chosen by the context's max_seq.
template <typename WT, int ROLE, int LPP, int MROWS, bool SPAN, bool LONGCTX>
__global__ __launch_bounds__(WG_THREADS, 1) void k_forward(FwdArgs args) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    Forward<WT, ROLE, LPP, MROWS, SPAN, LONGCTX> f(args, lds_raw);
    f.run();
}

}  // namespace sdfp
