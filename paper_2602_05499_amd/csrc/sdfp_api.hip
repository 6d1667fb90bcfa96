// Host side of libsdfp: context, argument / state / capacity checks, workspace layout and the launch
// sequences behind the C-ABI declared in include/sdfp.h (paper Sec. II-A, Alg. 1 Stage B, Sec. III-C).
#include "sdfp_kernels.hip.h"
#include "sdfp.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <type_traits>
#include <unordered_set>
#include <vector>

using namespace sdfp;

#define SDFP_EXTERN extern
#include "sdfp_inst.hip.h"

namespace {

enum Phase { PH_INIT = 0, PH_READY, PH_DRAFTED, PH_VERIFIED, PH_ACCEPTED };

struct Carve {   // byte offsets inside the workspace
    size_t state, out_tokens, prompt, cosT, sinT, h, q, att, a, part_o, part_ml, counters, zq, zp, head_val,
        head_idx, head_counter, layer_tab, skip_dev, bar, trace, total;
};

constexpr int HEAD_GRID_MAX = 1024;
constexpr int PREFILL_ROWS = 8;
constexpr int TRACE_CAP = 1024;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

bool config_ok(const sd_config* c) {
    if (!c) return false;
    if (c->n_layers < 1 || c->d_model < 8 || c->n_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 8 || c->vocab < 1)
        return false;
    if (c->head_dim < 8 || c->head_dim > 128 || (c->head_dim & (c->head_dim - 1))) return false;
    if (c->n_heads % c->n_kv_heads) return false;
    if (c->d_model % 8 || c->d_ffn % 8) return false;
    if (c->max_k < 0 || c->max_k > SD_MAX_K) return false;
    if (c->max_seq < c->max_k + 2) return false;
    if (c->dtype != SD_F32 && c->dtype != SD_BF16) return false;
    if (c->max_out < 1) return false;
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f) || !(c->temperature > 0.f)) return false;
    return true;
}

inline size_t esize(const sd_config* c) { return c->dtype == SD_F32 ? 4 : 2; }
inline int n_splits(const sd_config* c) { return (c->max_seq + ATT_SL - 1) / ATT_SL; }

Carve carve(const sd_config* c) {
    Carve k;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    const size_t dq = (size_t)c->n_heads * c->head_dim;
    k.state = take(sizeof(DevState));
    k.out_tokens = take(sizeof(int) * (size_t)c->max_out);
    k.prompt = take(sizeof(int) * (size_t)c->max_seq);
    k.cosT = take(sizeof(float) * (size_t)c->max_seq * (c->head_dim / 2));
    k.sinT = take(sizeof(float) * (size_t)c->max_seq * (c->head_dim / 2));
    k.h = take(sizeof(float) * MAX_ROWS * (size_t)c->d_model);
    k.q = take(sizeof(float) * MAX_ROWS * dq);
    k.att = take(sizeof(float) * MAX_ROWS * dq);
    k.a = take(sizeof(float) * MAX_ROWS * (size_t)c->d_ffn);
    k.part_o = take(sizeof(float) * (size_t)n_splits(c) * MAX_ROWS * dq);
    k.part_ml = take(sizeof(float) * (size_t)n_splits(c) * MAX_ROWS * c->n_heads * 2);
    k.counters = take(sizeof(unsigned) * (size_t)c->n_kv_heads);
    k.zq = take(sizeof(float) * (size_t)(c->max_k > 0 ? c->max_k : 1) * c->vocab);
    k.zp = take(sizeof(float) * (size_t)(c->max_k + 1) * c->vocab);
    k.head_val = take(sizeof(float) * HEAD_GRID_MAX * MAX_ROWS);
    k.head_idx = take(sizeof(int) * HEAD_GRID_MAX * MAX_ROWS);
    k.head_counter = take(sizeof(unsigned));
    k.layer_tab = take(sizeof(LayerW) * (size_t)c->n_layers);
    k.skip_dev = take((size_t)c->n_layers);
    k.bar = take(BAR_WORDS * sizeof(unsigned));
    k.trace = take(sizeof(unsigned long long) * (TRACE_CAP + 1));
    k.total = off;
    return k;
}

struct LayerPtrs {
    const float *attn_norm, *ffn_norm;
    const void *wq, *wk, *wv, *wo, *wg, *wu, *wd;
};

}  // namespace

struct sd_ctx {
    sd_config cfg;
    std::vector<LayerPtrs> layers;
    const void *tok_emb, *lm_head;
    const float* final_norm;
    std::vector<uint8_t> skip;
    char *kv, *ws;
    hipStream_t stream;
    Carve cv;
    Phase phase;
    bool dev_ready, keep_logits;
    int hip_err;
    int P_hi;        // upper bound of the device-side cache_len known to the host
    int out_hi;      // upper bound of the device-side committed count
    int K_cur, mode_cur;
    int n_cu;
    bool use_mega;        // whole forward in one persistent kernel (else one kernel per phase)
    unsigned spin_limit;  // bound of every grid-barrier wait, in polls
    bool trace_on;        // record workgroup 0's phase timeline of every forward
    std::unordered_set<const void*>* lds_set;

    DevState* st() const { return reinterpret_cast<DevState*>(ws + cv.state); }
    int* out_tokens() const { return reinterpret_cast<int*>(ws + cv.out_tokens); }
    int* prompt() const { return reinterpret_cast<int*>(ws + cv.prompt); }
    float* f(size_t off) const { return reinterpret_cast<float*>(ws + off); }
};

namespace {

#define HIPCHK(ctx, expr)                                   \
    do {                                                    \
        hipError_t e_ = (expr);                             \
        if (e_ != hipSuccess) {                             \
            (ctx)->hip_err = (int)e_;                       \
            if (std::getenv("SDFP_DEBUG"))                  \
                std::fprintf(stderr, "sdfp: %s -> %s (%s:%d)\n", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return SD_EHIP;                                 \
        }                                                   \
    } while (0)

template <class Kern>
int ensure_lds(sd_ctx* c, Kern kern, size_t bytes) {
    const void* key = reinterpret_cast<const void*>(kern);
    if (bytes > 48 * 1024 && !c->lds_set->count(key)) {
        HIPCHK(c, hipFuncSetAttribute(key, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
        c->lds_set->insert(key);
    }
    return SD_OK;
}

template <int N> using IC = std::integral_constant<int, N>;

// call fn(IC<MT>) with the smallest instantiated row count MT >= M
template <class Fn>
int dispatch_rows(int M, Fn&& fn) {
    switch (M) {
        case 1: return fn(IC<1>());
        case 2: return fn(IC<2>());
        case 3: return fn(IC<3>());
        case 4: return fn(IC<4>());
        case 5: return fn(IC<5>());
        case 6: return fn(IC<6>());
        case 7: return fn(IC<7>());
        case 8: return fn(IC<8>());
        case 9: return fn(IC<9>());
        default: return SD_EINVAL;
    }
}

template <typename WT>
int lazy_device_init(sd_ctx* c) {
    if (c->dev_ready) return SD_OK;
    const sd_config& g = c->cfg;
    const int half = g.head_dim / 2;
    std::vector<float> cs((size_t)g.max_seq * half), sn((size_t)g.max_seq * half);
    for (int p = 0; p < g.max_seq; ++p)
        for (int i = 0; i < half; ++i) {
            double ang = (double)p * std::pow((double)g.rope_theta, -2.0 * (double)i / (double)g.head_dim);
            cs[(size_t)p * half + i] = (float)std::cos(ang);
            sn[(size_t)p * half + i] = (float)std::sin(ang);
        }
    HIPCHK(c, hipMemcpyAsync(c->ws + c->cv.cosT, cs.data(), cs.size() * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(c->ws + c->cv.sinT, sn.data(), sn.size() * 4, hipMemcpyHostToDevice, c->stream));
    DevState z;
    std::memset(&z, 0, sizeof(z));
    z.max_out = g.max_out;
    HIPCHK(c, hipMemcpyAsync(c->st(), &z, sizeof(z), hipMemcpyHostToDevice, c->stream));
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(256), 0, c->stream,
                       reinterpret_cast<unsigned*>(c->ws + c->cv.counters), g.n_kv_heads);
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, c->stream,
                       reinterpret_cast<unsigned*>(c->ws + c->cv.head_counter), 1);
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, c->stream, reinterpret_cast<unsigned*>(c->ws + c->cv.bar), BAR_WORDS);
    std::vector<LayerW> tab(g.n_layers);
    for (int l = 0; l < g.n_layers; ++l) {
        const LayerPtrs& lp = c->layers[l];
        tab[l] = LayerW{lp.wq, lp.wk, lp.wv, lp.wo, lp.wg, lp.wu, lp.wd, lp.attn_norm, lp.ffn_norm};
    }
    HIPCHK(c, hipMemcpyAsync(c->ws + c->cv.layer_tab, tab.data(), tab.size() * sizeof(LayerW), hipMemcpyHostToDevice,
                             c->stream));
    HIPCHK(c, hipMemcpyAsync(c->ws + c->cv.skip_dev, c->skip.data(), c->skip.size(), hipMemcpyHostToDevice,
                             c->stream));
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipStreamSynchronize(c->stream));   // host vectors go out of scope
    int dev = 0;
    hipDeviceProp_t prop;
    HIPCHK(c, hipGetDevice(&dev));
    HIPCHK(c, hipGetDeviceProperties(&prop, dev));
    c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    if (c->n_cu > HEAD_GRID_MAX) c->n_cu = HEAD_GRID_MAX;
    const char* fw = std::getenv("SDFP_FORWARD");   // "split": one kernel per phase (debugging / comparison)
    c->use_mega = !(fw && std::strcmp(fw, "split") == 0);
    c->dev_ready = true;
    return SD_OK;
}

// where the output projection puts its result
struct HeadPlan {
    bool run;          // run the output projection at all
    int row_from;      // first row that gets logits (prefill: only the last row)
    float* logits;     // destination rows or nullptr
    int dst, off;      // ROWS_DRAFT -> st->d[off]; else st->amax[m]
};

template <typename WT>
int forward_mega(sd_ctx* c, Rows rows, bool use_skip, HeadPlan hp) {
    const sd_config& g = c->cfg;
    FwdArgs A;
    std::memset(&A, 0, sizeof(A));
    A.layers = reinterpret_cast<const LayerW*>(c->ws + c->cv.layer_tab);
    A.skip = use_skip ? reinterpret_cast<const unsigned char*>(c->ws + c->cv.skip_dev) : nullptr;
    A.n_layers = g.n_layers;
    A.L = LayerDims{g.d_model, g.n_heads, g.n_kv_heads, g.head_dim, g.d_ffn, g.vocab, g.max_seq};
    A.rows = rows;
    A.st = c->st();
    A.prompt = c->prompt();
    A.tok_emb = c->tok_emb; A.final_norm = c->final_norm; A.lm_head = c->lm_head;
    A.kv = c->kv;
    A.h = c->f(c->cv.h); A.q = c->f(c->cv.q); A.att = c->f(c->cv.att); A.a = c->f(c->cv.a);
    A.cosT = c->f(c->cv.cosT); A.sinT = c->f(c->cv.sinT);
    A.part_o = c->f(c->cv.part_o); A.part_ml = c->f(c->cv.part_ml);
    A.att_counters = reinterpret_cast<unsigned*>(c->ws + c->cv.counters);
    A.head.logits = hp.logits;
    A.head.part_val = c->f(c->cv.head_val);
    A.head.part_idx = reinterpret_cast<int*>(c->ws + c->cv.head_idx);
    A.head.counter = reinterpret_cast<unsigned*>(c->ws + c->cv.head_counter);
    A.head.dst = hp.dst; A.head.off = hp.off;
    A.head_run = hp.run ? 1 : 0;
    A.head_row_from = hp.run ? hp.row_from : 0;
    A.eps = g.rms_eps;
    A.bar = reinterpret_cast<unsigned*>(c->ws + c->cv.bar);
    A.spin_limit = c->spin_limit;
    A.trace = c->trace_on ? reinterpret_cast<unsigned long long*>(c->ws + c->cv.trace) : nullptr;
    A.trace_cap = TRACE_CAP;
    return dispatch_rows(rows.M, [&](auto mt) -> int {
        constexpr int MT = decltype(mt)::value;
        constexpr int D = ring_depth(MT);
        size_t lds = GEMV_LDS_BYTES;
        const size_t att_lds = attn_lds_bytes(g.head_dim);
        if (att_lds > lds) lds = att_lds;
        int e;
        if ((e = ensure_lds(c, k_forward<WT, MT, D>, lds))) return e;
        hipLaunchKernelGGL((k_forward<WT, MT, D>), dim3(c->n_cu), dim3(WG_THREADS), lds, c->stream, A);
        HIPCHK(c, hipGetLastError());
        return SD_OK;
    });
}

template <typename WT>
int forward_split(sd_ctx* c, Rows rows, bool use_skip, HeadPlan hp) {
    const sd_config& g = c->cfg;
    const int M = rows.M;
    LayerDims L{g.d_model, g.n_heads, g.n_kv_heads, g.head_dim, g.d_ffn, g.vocab, g.max_seq};
    float *h = c->f(c->cv.h), *q = c->f(c->cv.q), *att = c->f(c->cv.att), *a = c->f(c->cv.a);
    const float *cosT = c->f(c->cv.cosT), *sinT = c->f(c->cv.sinT);
    DevState* st = c->st();
    hipStream_t s = c->stream;
    const size_t plane = (size_t)g.n_kv_heads * g.max_seq * g.head_dim;   // elements per K or V plane

    {
        int gx = (g.d_model + 255) / 256;
        hipLaunchKernelGGL((k_embed<WT>), dim3(gx, M), dim3(256), 0, s, reinterpret_cast<const WT*>(c->tok_emb), h,
                           g.d_model, rows, st, c->prompt());
    }
    int rc = dispatch_rows(M, [&](auto mt) -> int {
        constexpr int MT = decltype(mt)::value;
        constexpr int D = ring_depth(MT);
        const size_t lds = GEMV_LDS_BYTES;
        int e;
        if ((e = ensure_lds(c, k_qkv<WT, MT, D>, lds))) return e;
        if ((e = ensure_lds(c, k_resid<WT, MT, D>, lds))) return e;
        if ((e = ensure_lds(c, k_gateup<WT, MT, D>, lds))) return e;
        const size_t att_lds = attn_lds_bytes(g.head_dim);
        if ((e = ensure_lds(c, k_attn<WT>, att_lds))) return e;
        const dim3 grid(c->n_cu), block(WG_THREADS);
        for (int l = 0; l < g.n_layers; ++l) {
            const LayerPtrs& lp = c->layers[l];
            const int sk = use_skip ? c->skip[l] : 0;
            if (!(sk & SD_SKIP_ATTN)) {
                WT* kc = reinterpret_cast<WT*>(c->kv) + (size_t)(2 * l) * plane;
                WT* vc = kc + plane;
                QkvOp<WT, MT> op;
                op.wq = (const WT*)lp.wq; op.wk = (const WT*)lp.wk; op.wv = (const WT*)lp.wv;
                op.kc = kc; op.vc = vc; op.q = q; op.cosT = cosT; op.sinT = sinT; op.L = L; op.M = M; op.pos0 = 0;
                hipLaunchKernelGGL((k_qkv<WT, MT, D>), grid, block, lds, s, op, rows, st, h, lp.attn_norm, g.rms_eps);
                AttnArgs aa;
                aa.q = q; aa.att = att; aa.part_o = c->f(c->cv.part_o); aa.part_ml = c->f(c->cv.part_ml);
                aa.counters = reinterpret_cast<unsigned*>(c->ws + c->cv.counters);
                aa.L = L; aa.rows = rows; aa.st = st;
                hipLaunchKernelGGL((k_attn<WT>), dim3(n_splits(&g), g.n_kv_heads), block, att_lds, s, kc, vc, aa);
                ResidOp<WT, MT> ro;
                ro.w = (const WT*)lp.wo; ro.h = h; ro.N = g.d_model; ro.K = g.n_heads * g.head_dim; ro.M = M;
                hipLaunchKernelGGL((k_resid<WT, MT, D>), grid, block, lds, s, ro, att);
            }
            if (!(sk & SD_SKIP_FFN)) {
                GateUpOp<WT, MT> go;
                go.wg = (const WT*)lp.wg; go.wu = (const WT*)lp.wu; go.a = a; go.F = g.d_ffn; go.d = g.d_model; go.M = M;
                hipLaunchKernelGGL((k_gateup<WT, MT, D>), grid, block, lds, s, go, h, lp.ffn_norm, g.rms_eps);
                ResidOp<WT, MT> ro;
                ro.w = (const WT*)lp.wd; ro.h = h; ro.N = g.d_model; ro.K = g.d_ffn; ro.M = M;
                hipLaunchKernelGGL((k_resid<WT, MT, D>), grid, block, lds, s, ro, a);
            }
        }
        return SD_OK;
    });
    if (rc) return rc;
    if (hp.run) {
        const int Mh = M - hp.row_from;
        rc = dispatch_rows(Mh, [&](auto mt) -> int {
            constexpr int MT = decltype(mt)::value;
            constexpr int D = ring_depth(MT);
            const size_t lds = GEMV_LDS_BYTES;
            int e;
            if ((e = ensure_lds(c, k_head<WT, MT, D>, lds))) return e;
            HeadOut ho;
            ho.logits = hp.logits;
            ho.part_val = c->f(c->cv.head_val);
            ho.part_idx = reinterpret_cast<int*>(c->ws + c->cv.head_idx);
            ho.counter = reinterpret_cast<unsigned*>(c->ws + c->cv.head_counter);
            ho.dst = hp.dst; ho.off = hp.off;
            hipLaunchKernelGGL((k_head<WT, MT, D>), dim3(c->n_cu), dim3(WG_THREADS), lds, s, (const WT*)c->lm_head,
                               h + (size_t)hp.row_from * g.d_model, c->final_norm, g.rms_eps, g.vocab, g.d_model, Mh,
                               ho, st);
            return SD_OK;
        });
        if (rc) return rc;
    }
    HIPCHK(c, hipGetLastError());
    return SD_OK;
}

template <typename WT>
int forward(sd_ctx* c, Rows rows, bool use_skip, HeadPlan hp) {
    return c->use_mega ? forward_mega<WT>(c, rows, use_skip, hp) : forward_split<WT>(c, rows, use_skip, hp);
}

template <typename WT>
int do_prefill(sd_ctx* c, const int32_t* prompt_host, int n, int mode, const float* u_host) {
    int e = lazy_device_init<WT>(c);
    if (e) return e;
    HIPCHK(c, hipMemcpyAsync(c->prompt(), prompt_host, sizeof(int) * (size_t)n, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));   // prompt_host may be reused by the caller on return
    for (int p0 = 0; p0 < n; p0 += PREFILL_ROWS) {
        Rows rows{std::min(PREFILL_ROWS, n - p0), ROWS_PROMPT, p0};
        const bool last = p0 + PREFILL_ROWS >= n;
        HeadPlan hp{last, rows.M - 1, c->f(c->cv.zp), ROWS_VERIFY, 0};
        if (last && !(mode == SD_SAMPLE || c->keep_logits)) hp.logits = nullptr;
        if ((e = forward<WT>(c, rows, false, hp))) return e;
    }
    if (mode == SD_SAMPLE)
        hipLaunchKernelGGL(k_pick_sample, dim3(1), dim3(1024), 0, c->stream, c->f(c->cv.zp), c->cfg.vocab,
                           c->cfg.temperature, u_host[0], c->st(), (int)ROWS_VERIFY, 0);
    hipLaunchKernelGGL(k_commit_first, dim3(1), dim3(64), 0, c->stream, c->st(), c->out_tokens(), n);
    HIPCHK(c, hipGetLastError());
    return SD_OK;
}

template <typename WT>
int do_draft(sd_ctx* c, int K, int mode, const float* u_host) {
    hipLaunchKernelGGL(k_set_k, dim3(1), dim3(64), 0, c->stream, c->st(), K);
    for (int i = 0; i < K; ++i) {
        Rows rows{1, ROWS_DRAFT, i};
        const bool keep = (mode == SD_SAMPLE) || c->keep_logits;
        HeadPlan hp{true, 0, keep ? c->f(c->cv.zq) + (size_t)i * c->cfg.vocab : nullptr, ROWS_DRAFT, i};
        int e = forward<WT>(c, rows, true, hp);
        if (e) return e;
        if (mode == SD_SAMPLE)
            hipLaunchKernelGGL(k_pick_sample, dim3(1), dim3(1024), 0, c->stream,
                               c->f(c->cv.zq) + (size_t)i * c->cfg.vocab, c->cfg.vocab, c->cfg.temperature, u_host[i],
                               c->st(), (int)ROWS_DRAFT, i);
    }
    HIPCHK(c, hipGetLastError());
    return SD_OK;
}

template <typename WT>
int do_verify(sd_ctx* c) {
    Rows rows{c->K_cur + 1, ROWS_VERIFY, 0};
    const bool keep = (c->mode_cur == SD_SAMPLE) || c->keep_logits;
    HeadPlan hp{true, 0, keep ? c->f(c->cv.zp) : nullptr, ROWS_VERIFY, 0};
    return forward<WT>(c, rows, false, hp);
}

int do_accept(sd_ctx* c, int mode, const float* u_host) {
    if (mode == SD_GREEDY) {
        hipLaunchKernelGGL(k_accept_greedy, dim3(1), dim3(64), 0, c->stream, c->st(), c->out_tokens());
    } else {
        Uni un;
        std::memset(&un, 0, sizeof(un));
        for (int i = 0; i <= c->K_cur; ++i) un.u[i] = u_host[i];
        hipLaunchKernelGGL(k_accept_sample, dim3(1), dim3(1024), 0, c->stream, c->f(c->cv.zq), c->f(c->cv.zp),
                           c->cfg.vocab, c->cfg.temperature, un, c->st(), c->out_tokens());
    }
    HIPCHK(c, hipGetLastError());
    return SD_OK;
}

// refresh the host-side bounds from the device state (synchronises)
int refresh_bounds(sd_ctx* c, DevState* out) {
    DevState z;
    HIPCHK(c, hipMemcpyAsync(&z, c->st(), sizeof(z), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    // P and n_out on the device already include every enqueued rollback / commit
    c->P_hi = z.P + ((c->phase == PH_ACCEPTED) ? z.n_acc + 1 : 0);
    c->out_hi = z.n_out;
    if (out) *out = z;
    return SD_OK;
}

int check_capacity(sd_ctx* c, int K) {
    if (c->P_hi + K + 1 > c->cfg.max_seq || c->out_hi + K + 1 > c->cfg.max_out) {
        int e = refresh_bounds(c, nullptr);   // the bound may be stale: get the exact values once
        if (e) return e;
        if (c->P_hi + K + 1 > c->cfg.max_seq || c->out_hi + K + 1 > c->cfg.max_out) return SD_ECAPACITY;
    }
    return SD_OK;
}

bool mode_ok(int mode) { return mode == SD_GREEDY || mode == SD_SAMPLE; }

}  // namespace

#define DT_CALL(ctx, fn, ...) ((ctx)->cfg.dtype == SD_F32 ? fn<float>(__VA_ARGS__) : fn<bf16_t>(__VA_ARGS__))

extern "C" {

size_t sd_kv_bytes(const sd_config* cfg) {
    if (!config_ok(cfg)) return 0;
    return align_up((size_t)cfg->n_layers * 2 * cfg->n_kv_heads * cfg->max_seq * cfg->head_dim * esize(cfg));
}

size_t sd_workspace_bytes(const sd_config* cfg) {
    if (!config_ok(cfg)) return 0;
    return carve(cfg).total;
}

int sd_init(sd_ctx** out, const sd_config* cfg, const sd_weights* w, const uint8_t* skip_mask, void* kv_buf,
            size_t kv_bytes, void* ws_buf, size_t ws_bytes, void* hip_stream) {
    if (!out) return SD_EINVAL;
    *out = nullptr;
    if (!config_ok(cfg) || !w || !kv_buf || !ws_buf) return SD_EINVAL;
    if (((uintptr_t)kv_buf | (uintptr_t)ws_buf) & 255) return SD_EINVAL;
    if (!w->tok_emb || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo ||
        !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
        return SD_EINVAL;
    if (((uintptr_t)w->tok_emb | (uintptr_t)w->lm_head | (uintptr_t)w->final_norm) & 15) return SD_EINVAL;
    for (int l = 0; l < cfg->n_layers; ++l) {
        const void* ps[9] = {w->attn_norm[l], w->wq[l], w->wk[l], w->wv[l], w->wo[l],
                             w->ffn_norm[l], w->w_gate[l], w->w_up[l], w->w_down[l]};
        for (const void* p : ps)
            if (!p || ((uintptr_t)p & 15)) return SD_EINVAL;
    }
    if (kv_bytes < sd_kv_bytes(cfg) || ws_bytes < sd_workspace_bytes(cfg)) return SD_ENOMEM;
    sd_ctx* c = new (std::nothrow) sd_ctx();
    if (!c) return SD_ENOMEM;
    c->cfg = *cfg;
    c->layers.resize(cfg->n_layers);
    for (int l = 0; l < cfg->n_layers; ++l)
        c->layers[l] = LayerPtrs{w->attn_norm[l], w->ffn_norm[l], w->wq[l], w->wk[l], w->wv[l],
                                 w->wo[l], w->w_gate[l], w->w_up[l], w->w_down[l]};
    c->tok_emb = w->tok_emb; c->lm_head = w->lm_head; c->final_norm = w->final_norm;
    c->skip.assign(cfg->n_layers, 0);
    if (skip_mask)
        for (int l = 0; l < cfg->n_layers; ++l) c->skip[l] = skip_mask[l] & 3;
    c->kv = (char*)kv_buf; c->ws = (char*)ws_buf;
    c->stream = (hipStream_t)hip_stream;
    c->cv = carve(cfg);
    c->phase = PH_INIT;
    c->dev_ready = false; c->keep_logits = false;
    c->hip_err = 0; c->P_hi = 0; c->out_hi = 0; c->K_cur = 0; c->mode_cur = SD_GREEDY; c->n_cu = 256;
    c->use_mega = true; c->spin_limit = 1u << 21; c->trace_on = false;
    c->lds_set = new std::unordered_set<const void*>();
    *out = c;
    return SD_OK;
}

int sd_set_skip_mask(sd_ctx* c, const uint8_t* skip_mask) {
    if (!c || !skip_mask) return SD_EINVAL;
    if (c->phase == PH_DRAFTED) return SD_ESTATE;   // a drafted block must be verified with the mask it used
    for (int l = 0; l < c->cfg.n_layers; ++l) c->skip[l] = skip_mask[l] & 3;
    if (c->dev_ready) {
        HIPCHK(c, hipMemcpyAsync(c->ws + c->cv.skip_dev, c->skip.data(), c->skip.size(), hipMemcpyHostToDevice,
                                 c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
    }
    return SD_OK;
}

int sd_prefill(sd_ctx* c, const int32_t* prompt_host, int32_t n, int mode, const float* u_host) {
    if (!c || !prompt_host || n < 1 || !mode_ok(mode)) return SD_EINVAL;
    if (mode == SD_SAMPLE && (!u_host || !(u_host[0] >= 0.f && u_host[0] < 1.f))) return SD_EINVAL;
    if (n + c->cfg.max_k + 1 > c->cfg.max_seq) return SD_ECAPACITY;
    for (int i = 0; i < n; ++i)
        if (prompt_host[i] < 0 || prompt_host[i] >= c->cfg.vocab) return SD_EINVAL;
    int e = DT_CALL(c, do_prefill, c, prompt_host, n, mode, u_host);
    if (e) return e;
    c->phase = PH_READY;
    c->P_hi = n; c->out_hi = 1; c->K_cur = 0; c->mode_cur = mode;
    return SD_OK;
}

int sd_draft(sd_ctx* c, int32_t K, int mode, const float* u_host) {
    if (!c || !mode_ok(mode) || K < 0 || K > c->cfg.max_k) return SD_EINVAL;
    if (c->phase != PH_READY) return SD_ESTATE;
    if (mode == SD_SAMPLE) {
        if (K > 0 && !u_host) return SD_EINVAL;
        for (int i = 0; i < K; ++i)
            if (!(u_host[i] >= 0.f && u_host[i] < 1.f)) return SD_EINVAL;
    }
    int e = check_capacity(c, K);
    if (e) return e;
    e = DT_CALL(c, do_draft, c, K, mode, u_host);
    if (e) return e;
    c->K_cur = K; c->mode_cur = mode;
    c->phase = PH_DRAFTED;
    return SD_OK;
}

int sd_verify(sd_ctx* c) {
    if (!c) return SD_EINVAL;
    if (c->phase != PH_DRAFTED) return SD_ESTATE;
    int e = DT_CALL(c, do_verify, c);
    if (e) return e;
    c->phase = PH_VERIFIED;
    return SD_OK;
}

int sd_accept(sd_ctx* c, int mode, const float* u_host) {
    if (!c || !mode_ok(mode)) return SD_EINVAL;
    if (c->phase != PH_VERIFIED) return SD_ESTATE;
    if (mode != c->mode_cur) return SD_EINVAL;
    if (mode == SD_SAMPLE) {
        if (!u_host) return SD_EINVAL;
        for (int i = 0; i <= c->K_cur; ++i)
            if (!(u_host[i] >= 0.f && u_host[i] < 1.f)) return SD_EINVAL;
    }
    int e = do_accept(c, mode, u_host);
    if (e) return e;
    c->out_hi += c->K_cur + 1;
    c->phase = PH_ACCEPTED;
    return SD_OK;
}

int sd_rollback(sd_ctx* c) {
    if (!c) return SD_EINVAL;
    if (c->phase != PH_ACCEPTED) return SD_ESTATE;
    hipLaunchKernelGGL(k_rollback, dim3(1), dim3(64), 0, c->stream, c->st());
    HIPCHK(c, hipGetLastError());
    c->P_hi += c->K_cur + 1;
    c->phase = PH_READY;
    return SD_OK;
}

int sd_decode(sd_ctx* c, int mode, const float* u_host) {
    if (!c || !mode_ok(mode)) return SD_EINVAL;
    if (mode == SD_SAMPLE && !u_host) return SD_EINVAL;
    int e = sd_draft(c, 0, mode, nullptr);
    if (e) return e;
    if ((e = sd_verify(c))) return e;
    if ((e = sd_accept(c, mode, u_host))) return e;
    return sd_rollback(c);
}

int sd_set_pending(sd_ctx* c, int32_t cache_len, int32_t token) {
    if (!c || token < 0 || token >= c->cfg.vocab || cache_len < 1) return SD_EINVAL;
    if (c->phase != PH_READY) return SD_ESTATE;
    if (cache_len + 1 > c->cfg.max_seq) return SD_ECAPACITY;
    hipLaunchKernelGGL(k_set_pending, dim3(1), dim3(64), 0, c->stream, c->st(), cache_len, token);
    HIPCHK(c, hipGetLastError());
    c->P_hi = cache_len;
    return SD_OK;
}

int sd_set_draft(sd_ctx* c, const int32_t* d_host, int32_t K) {
    if (!c || K < 0 || K > c->cfg.max_k || (K > 0 && !d_host)) return SD_EINVAL;
    if (c->phase != PH_READY && c->phase != PH_DRAFTED) return SD_ESTATE;
    DraftBlock b;
    std::memset(&b, 0, sizeof(b));
    for (int i = 0; i < K; ++i) {
        if (d_host[i] < 0 || d_host[i] >= c->cfg.vocab) return SD_EINVAL;
        b.d[i] = d_host[i];
    }
    int e = check_capacity(c, K);
    if (e) return e;
    hipLaunchKernelGGL(k_set_draft, dim3(1), dim3(64), 0, c->stream, c->st(), b, K);
    HIPCHK(c, hipGetLastError());
    c->K_cur = K;
    if (c->phase == PH_READY) c->mode_cur = SD_GREEDY;
    c->phase = PH_DRAFTED;
    return SD_OK;
}

int sd_read(sd_ctx* c, int32_t* tokens_host, int32_t cap, int32_t* n_committed, sd_stats* stats) {
    if (!c || cap < 0 || (cap > 0 && !tokens_host)) return SD_EINVAL;
    if (c->phase == PH_INIT) return SD_ESTATE;
    DevState z;
    int e = refresh_bounds(c, &z);
    if (e) return e;
    unsigned flag = 0;
    HIPCHK(c, hipMemcpyAsync(&flag, c->ws + c->cv.bar + BAR_STRIDE * sizeof(unsigned), sizeof(flag),
                             hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (flag != 0) return SD_ETIMEOUT;
    int n = z.n_out < cap ? z.n_out : cap;
    if (n > 0) {
        HIPCHK(c, hipMemcpyAsync(tokens_host, c->out_tokens(), sizeof(int) * (size_t)n, hipMemcpyDeviceToHost,
                                 c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
    }
    if (n_committed) *n_committed = z.n_out;
    if (stats) {
        stats->steps = z.steps; stats->drafted = z.drafted; stats->accepted = z.accepted;
        stats->examined = z.examined; stats->committed = z.n_out; stats->cache_len = z.P;
        stats->t_last = z.t_last; stats->last_n = z.n_acc; stats->last_k = z.K;
    }
    return SD_OK;
}

int sd_dump_logits(sd_ctx* c, int which, float* host, size_t cap) {
    if (!c || !host || (which != SD_LOGITS_DRAFT && which != SD_LOGITS_VERIFY)) return SD_EINVAL;
    if (c->phase == PH_INIT) return SD_ESTATE;
    size_t rows = which == SD_LOGITS_DRAFT ? (size_t)c->K_cur : (size_t)c->K_cur + 1;
    size_t n = rows * (size_t)c->cfg.vocab;
    if (cap < n) return SD_EINVAL;
    if (n == 0) return SD_OK;
    HIPCHK(c, hipMemcpyAsync(host, c->f(which == SD_LOGITS_DRAFT ? c->cv.zq : c->cv.zp), n * sizeof(float),
                             hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return SD_OK;
}

int sd_dump_draft(sd_ctx* c, int32_t* d_host, int32_t cap) {
    if (!c || !d_host || cap < c->K_cur) return SD_EINVAL;
    if (c->phase == PH_INIT) return SD_ESTATE;
    DevState z;
    HIPCHK(c, hipMemcpyAsync(&z, c->st(), sizeof(z), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    for (int i = 0; i < c->K_cur; ++i) d_host[i] = z.d[i];
    return SD_OK;
}

int sd_keep_logits(sd_ctx* c, int on) {
    if (!c) return SD_EINVAL;
    c->keep_logits = on != 0;
    return SD_OK;
}

int sd_phase_trace(sd_ctx* c, int on) {
    if (!c) return SD_EINVAL;
    c->trace_on = on != 0;
    return SD_OK;
}

int sd_phase_trace_read(sd_ctx* c, uint64_t* host, int32_t cap, int32_t* n) {
    if (!c || !host || cap < 0 || !n) return SD_EINVAL;
    if (!c->dev_ready) return SD_ESTATE;
    std::vector<unsigned long long> buf(TRACE_CAP + 1);
    HIPCHK(c, hipMemcpyAsync(buf.data(), c->ws + c->cv.trace, buf.size() * sizeof(unsigned long long),
                             hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    int cnt = (int)buf[TRACE_CAP];
    if (cnt < 0 || cnt > TRACE_CAP) cnt = 0;
    *n = cnt;
    for (int i = 0; i < cnt && i < cap; ++i) host[i] = buf[i];
    return SD_OK;
}

int sd_sync(sd_ctx* c) {
    if (!c) return SD_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return SD_OK;
}

int sd_last_hip_error(const sd_ctx* c) { return c ? c->hip_err : 0; }

void sd_free(sd_ctx* c) {
    if (!c) return;
    delete c->lds_set;
    delete c;
}

const char* sd_strerror(int code) {
    switch (code) {
        case SD_OK: return "ok";
        case SD_EINVAL: return "invalid argument";
        case SD_ECAPACITY: return "KV cache or output list capacity exceeded";
        case SD_ESTATE: return "call out of order";
        case SD_EHIP: return "HIP runtime error";
        case SD_ENOMEM: return "buffer too small";
        case SD_ETIMEOUT: return "a grid barrier of the forward kernel timed out (workgroups not co-resident)";
        default: return "unknown error";
    }
}

}  // extern "C"
