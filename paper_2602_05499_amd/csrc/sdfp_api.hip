// Host side of libsdfp: context, argument / state / capacity checks, workspace layout and the launch
// sequences behind the C-ABI declared in include/sdfp.h (paper Sec. II-A, Alg. 1 Stage B, Sec. III-C).
#include "sdfp_kernels.hip.h"
#include "sdfp_prefill.hip.h"
#include "sdfp.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

using namespace sdfp;

// The forward kernels are instantiated in the sdfp_fwd_<type>_hd<n>.hip translation units: per storage type and
// head_dim, one for prompt chunks, one draft row, one plain decode row, and one verify kernel per row count 2..9.
namespace sdfp {
#define SDFP_DECL(WT, ROLE, LPP, M, SPAN, LC) extern template __global__ void k_forward<WT, ROLE, LPP, M, SPAN, LC>(FwdArgs);
#define SDFP_DECL_DECODE(WT, LPP, SPAN, LC)                                                                       \
    SDFP_DECL(WT, 1, LPP, 1, SPAN, LC) SDFP_DECL(WT, 3, LPP, 1, SPAN, LC)                                          \
    SDFP_DECL(WT, 2, LPP, 2, SPAN, LC) SDFP_DECL(WT, 2, LPP, 3, SPAN, LC) SDFP_DECL(WT, 2, LPP, 4, SPAN, LC)       \
    SDFP_DECL(WT, 2, LPP, 5, SPAN, LC) SDFP_DECL(WT, 2, LPP, 6, SPAN, LC) SDFP_DECL(WT, 2, LPP, 7, SPAN, LC)       \
    SDFP_DECL(WT, 2, LPP, 8, SPAN, LC) SDFP_DECL(WT, 2, LPP, 9, SPAN, LC)
#define SDFP_DECL_HD(WT, LPP)                                                                                       \
    SDFP_DECL(WT, 0, LPP, 0, false, true) SDFP_DECL_DECODE(WT, LPP, false, false) SDFP_DECL_DECODE(WT, LPP, true, false) \
    SDFP_DECL_DECODE(WT, LPP, false, true) SDFP_DECL_DECODE(WT, LPP, true, true)
SDFP_DECL_HD(float, 4) SDFP_DECL_HD(float, 8) SDFP_DECL_HD(float, 16) SDFP_DECL_HD(float, 32)
SDFP_DECL_HD(bf16_t, 4) SDFP_DECL_HD(bf16_t, 8) SDFP_DECL_HD(bf16_t, 16) SDFP_DECL_HD(bf16_t, 32)
#undef SDFP_DECL_HD
#undef SDFP_DECL_DECODE
#undef SDFP_DECL
static_assert(MAX_K + 1 == 9, "one verify kernel per row count up to MAX_K + 1");
}  // namespace sdfp


namespace {

enum StepState { PH_INIT = 0, PH_READY, PH_DRAFTED, PH_VERIFIED, PH_ACCEPTED };

struct Carve {   // byte offsets inside the workspace
    size_t state, out_tokens, prompt, cosT, sinT, acts, part_o, part_ml, counters, zq, zp, head_val, head_idx,
        prog_target, prog_draft, prog_head, bar, trace, guard_rec, total;
    size_t act_h, act_q, act_a;   // bytes of one residual / query / feed-forward activation block
    size_t acts_bytes;            // bytes of the activation region (also the scratch of the matrix-matrix prompt path)
};

constexpr int HEAD_GRID_MAX = 1024;
constexpr int PREFILL_ROWS = MAX_ROWS;
// shortest prompt that goes through the matrix-matrix path by default: on the 7B shape that path takes 4.1 ms for 4 rows,
// 4.2 (8), 4.6 (16), 5.2 (32), 6.5 (64); the 16-row forward 3.3 ms (1 row), 3.8 (4), 4.6 (6), 5.0 (8), 10.5 (16)
constexpr int PREFILL_MATRIX_MIN_ROWS = 5;
constexpr int TRACE_CAP = 1024;
constexpr int LDS_DONE_MAX = 64;   // a context launches at most 3 + 2 * 8 different forward kernels and some 25 of the prompt path

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

bool config_ok(const sd_config* c) {
    if (!c) return false;
    if (c->n_layers < 1 || c->d_model < 8 || c->n_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 8 || c->vocab < 1)
        return false;
    if (c->head_dim < 16 || c->head_dim > 128 || (c->head_dim & (c->head_dim - 1))) return false;
    if (c->n_heads % c->n_kv_heads) return false;
    // the query vectors of one KV head's group, for the largest forward, are kept in LDS by the attention phase
    if (attn_lds_bytes(c->head_dim, MAX_ROWS * (c->n_heads / c->n_kv_heads)) > (size_t)LDS_ZERO_OFF) return false;
    if (c->dtype != SD_F32 && c->dtype != SD_BF16) return false;
    // a weight row is consumed in 64-byte steps
    const int q = c->dtype == SD_F32 ? 16 : 32;
    if (c->d_model % q || c->d_ffn % q || (c->n_heads * c->head_dim) % q) return false;
    if (c->max_k < 0 || c->max_k > SD_MAX_K) return false;
    if (c->max_seq < c->max_k + 2) return false;
    if (c->max_out < 1) return false;
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f) || !(c->temperature > 0.f)) return false;
    return true;
}

inline size_t esize(const sd_config* c) { return c->dtype == SD_F32 ? 4 : 2; }

// A turn of the register ring holds four 2 KB blocks of one 16-row tile.  The kernels whose turns may go on into the
// next tile pay a few scalar operations per load for it, so they are used only where they gain: where the blocks of
// a weight row do not fill whole turns and a workgroup has more than one tile of such rows to go on into.
inline bool span_pays(const sd_config* c, int n_wg) {
    const int turn = RING_MAX / SPW;
    auto ragged = [&](int Kd) { return (int)(((size_t)Kd * esize(c) + BLOCK_BYTES - 1) / BLOCK_BYTES) % turn != 0; };
    const int hq = c->n_heads * c->head_dim, hkv = c->n_kv_heads * c->head_dim;
    const bool many_d_rows = c->d_model / 16 > n_wg;   // O and down projection: tiles per workgroup > 1
    const bool many_x_rows = (hq + 2 * hkv) / 16 > n_wg || c->d_ffn / 8 > n_wg || c->vocab / 16 > n_wg;
    return (ragged(c->d_model) && many_x_rows) || ((ragged(hq) || ragged(c->d_ffn)) && many_d_rows);
}
inline int n_splits(const sd_config* c) { return (c->max_seq + ATT_SL - 1) / ATT_SL; }
inline size_t prog_len(const sd_config* c) { return (size_t)c->n_layers * 5 + 3; }

// The matrix-matrix prompt path works on panels of P prompt rows whose buffers live in the workspace's activation
// region (no forward of the decode kind runs meanwhile).  Byte offsets from the region's start.
struct PanelPlan {
    int P;                 // rows per panel (a multiple of 64), 0 = the path is not available for this configuration
    int n_awg;             // workgroups of the panel's attention kernel (each owns a region of split partials)
    size_t h_last, h, q, att, rs, xs_a, xs_b, shares, part, counters;
    size_t part_stride;    // floats per attention workgroup region
    size_t part_ml_off;    // floats from a region's start to its (max, sum) pairs
    int Ka;                // row length of xs_a: max(d_model, n_heads * head_dim)
};
constexpr int PANEL_MAX_ROWS = 512, PANEL_MAX_AWG = 512;   // (two attention workgroups per compute unit)
constexpr size_t PANEL_MAX_BYTES = (size_t)1 << 30;   // a workspace never grows past this for the sake of a larger panel
// bytes per panel row: residual stream, queries, attention output, reciprocal RMS, the pieces of the two projection
// inputs, and the 8 per-share partial sums of an O / down projection
inline size_t panel_row_bytes(const sd_config* c) {
    const size_t d = c->d_model, hq = (size_t)c->n_heads * c->head_dim, F = c->d_ffn;
    return d * 4 + 2 * hq * 4 + 4 + 6 * std::max(d, hq) + 6 * F + PF_NSHARE * d * 4;
}
inline size_t panel_region_floats(const sd_config* c) {   // split partials of one attention workgroup
    const size_t grp = c->n_heads / c->n_kv_heads, n_spl = (c->max_seq + ATT_SL - 1) / ATT_SL;
    return n_spl * MAX_ROWS * grp * (c->head_dim + 2);
}
inline size_t panel_bytes(const sd_config* c, int P, int n_awg) {
    return align_up((size_t)c->d_model * 4) + 16 * 256 + PANEL_MAX_AWG * 4 + 1024 + (size_t)P * panel_row_bytes(c) +
           (size_t)n_awg * panel_region_floats(c) * 4;
}
PanelPlan plan_panel(const sd_config* c, size_t region_bytes) {
    PanelPlan pl;
    std::memset(&pl, 0, sizeof(pl));
    if (c->dtype != SD_BF16) return pl;
    const size_t d = c->d_model, hq = (size_t)c->n_heads * c->head_dim, F = c->d_ffn;
    const size_t grp = c->n_heads / c->n_kv_heads, n_spl = (c->max_seq + ATT_SL - 1) / ATT_SL;
    pl.Ka = (int)std::max(d, hq);
    pl.part_ml_off = n_spl * MAX_ROWS * grp * c->head_dim;
    pl.part_stride = panel_region_floats(c);
    const size_t region = pl.part_stride * 4;
    for (int want : {64, 8}) {
        for (int P = PANEL_MAX_ROWS; P >= 64; P -= 64) {
            const size_t need = panel_bytes(c, P, 0);
            if (need > region_bytes) continue;
            const size_t n_awg = std::min<size_t>(PANEL_MAX_AWG, (region_bytes - need) / region);
            if ((int)n_awg < want) continue;
            pl.P = P; pl.n_awg = (int)n_awg;
            size_t off = 0;
            auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
            pl.h_last = take(d * 4);
            pl.h = take((size_t)P * d * 4); pl.q = take((size_t)P * hq * 4); pl.att = take((size_t)P * hq * 4);
            pl.rs = take((size_t)P * 4);
            pl.xs_a = take((size_t)3 * P * pl.Ka * 2); pl.xs_b = take((size_t)3 * P * F * 2);
            pl.shares = take((size_t)PF_NSHARE * P * d * 4);
            pl.counters = take(PANEL_MAX_AWG * 4);
            pl.part = take((size_t)pl.n_awg * region);
            if (off > region_bytes) { pl.P = 0; continue; }
            return pl;
        }
    }
    pl.P = 0;
    return pl;
}
// the activation region the workspace asks for on behalf of the prompt path: a full panel if that stays under the
// cap, else whatever the cap allows (plan_panel then settles for fewer rows), never less than 64 rows and 8 regions.
// compact: only that minimum (the static workspace is small; plan_panel uses what the decode kernels' buffers leave)
size_t panel_want_bytes(const sd_config* c, bool compact) {
    if (c->dtype != SD_BF16) return 0;
    const size_t least = panel_bytes(c, 64, 8);
    if (compact) return least;
    return std::max(least, std::min(panel_bytes(c, PANEL_MAX_ROWS, PANEL_MAX_AWG), PANEL_MAX_BYTES));
}

Carve carve(const sd_config* c, bool compact = false) {
    Carve k;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    const size_t dq = (size_t)c->n_heads * c->head_dim;
    k.state = take(sizeof(DevState));
    k.out_tokens = take(sizeof(int) * (size_t)c->max_out);
    k.prompt = take(sizeof(int) * (size_t)c->max_seq);
    k.cosT = take(sizeof(float) * (size_t)c->max_seq * (c->head_dim / 2));
    k.sinT = take(sizeof(float) * (size_t)c->max_seq * (c->head_dim / 2));
    // activations: every buffer is written once per forward (see sdfp_forward.hip.h).  Layout: the embedding
    // output, then per layer { q, attention output, residual after attention, feed-forward activation,
    // residual after the feed-forward }.
    k.act_h = align_up(sizeof(float) * MAX_ROWS * (size_t)c->d_model);
    k.act_q = align_up(sizeof(float) * MAX_ROWS * dq);
    k.act_a = align_up(sizeof(float) * MAX_ROWS * (size_t)c->d_ffn);
    k.acts_bytes = std::max(k.act_h + (size_t)c->n_layers * (2 * k.act_q + 2 * k.act_h + k.act_a), panel_want_bytes(c, compact));
    k.acts = take(k.acts_bytes);
    k.part_o = take(sizeof(float) * (size_t)n_splits(c) * MAX_ROWS * dq);
    k.part_ml = take(sizeof(float) * (size_t)n_splits(c) * MAX_ROWS * c->n_heads * 2);
    k.counters = take(sizeof(unsigned) * (size_t)c->n_kv_heads);
    k.zq = take(sizeof(float) * (size_t)(c->max_k > 0 ? c->max_k : 1) * c->vocab);
    k.zp = take(sizeof(float) * (size_t)(c->max_k + 1) * c->vocab);
    k.head_val = take(sizeof(float) * HEAD_GRID_MAX * MAX_ROWS);
    k.head_idx = take(sizeof(int) * HEAD_GRID_MAX * MAX_ROWS);
    k.prog_target = take(sizeof(Phase) * prog_len(c));
    k.prog_draft = take(sizeof(Phase) * prog_len(c));
    k.prog_head = take(sizeof(Phase) * 2);   // the output head alone, for the prompt's last row (matrix-matrix prompt path)
    k.bar = take(BAR_WORDS * sizeof(unsigned));
    k.trace = take(sizeof(unsigned long long) * (TRACE_CAP + 1));
    k.guard_rec = take(sizeof(unsigned long long) * 32);
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
    LayerPtrs* layers;   // [n_layers]; the context's own storage (heap, or the static slot's arrays)
    const void *tok_emb, *lm_head;
    const float* final_norm;
    uint8_t* skip;       // [n_layers]
    char *kv, *ws;
    hipStream_t stream;
    Carve cv;
    StepState phase;
    bool dev_ready, keep_logits;
    int hip_err;
    int P_hi;        // upper bound of the device-side cache_len known to the host
    int out_hi;      // upper bound of the device-side committed count
    int K_cur, mode_cur;
    int n_cu;
    unsigned spin_limit;  // bound of every grid-barrier and hand-over wait, in polls
    int n_prog[2];        // entries of the target / draft phase list
    bool span;            // use the kernels whose ring turns go on into the next tile (see span_pays)
    int span_mode;        // -1 = decide from the shapes, 0 / 1 = forced by sd_set_turn_span
    bool trace_on;        // record workgroup 0's phase timeline of every forward
    const void* lds_done[LDS_DONE_MAX];   // kernels whose dynamic-LDS limit has been raised and whose occupancy is checked
    int n_lds_done;
    int static_dev;       // device whose static workspace this context uses, or -1 (caller's workspace)
    int prefill_mode;     // -1 = choose (matrix-matrix path for bf16 prompts of PREFILL_MATRIX_MIN_ROWS or more), 0 = 16-row chunks, 1 = matrix-matrix
    PanelPlan panel;      // layout of a prompt panel inside the activation region (matrix-matrix prompt path)
    const char* tiled;    // the layer matrices in the prompt path's tile order (sd_set_tiled_weights), or nullptr
    const char *w_lo, *w_hi;   // address range spanned by the weight tensors (guard build)
    unsigned long long* dbg_host;   // pinned host buffer for guard records and beacons (guard build), or nullptr

    DevState* st() const { return reinterpret_cast<DevState*>(ws + cv.state); }
    int* out_tokens() const { return reinterpret_cast<int*>(ws + cv.out_tokens); }
    int* prompt() const { return reinterpret_cast<int*>(ws + cv.prompt); }
    float* f(size_t off) const { return reinterpret_cast<float*>(ws + off); }
};

// ---- the workspace of contexts made by sd_init_static: device memory that belongs to the library image ------------
// One array per GPU (every device that loads the library holds its own copy at its own address until the process
// ends).  In host code the array's name is only a handle for hipGetSymbolAddress: the address that kernels, copies
// and fills use is the one that call returns for the current device, kept in g_static[device].ws.
static __device__ __align__(256) unsigned char scratch[SD_STATIC_WS_BYTES];

namespace {
constexpr int STATIC_MAX_DEVICES = 16;
struct StaticSlot {
    void* ws;                                  // device address of `scratch` on this device, once resolved
    bool in_use;                               // a context made by sd_init_static on this device is alive
    sd_ctx ctx;                                // that context, and the arrays it points to
    LayerPtrs layers[SD_STATIC_MAX_LAYERS];
    uint8_t skip[SD_STATIC_MAX_LAYERS];
};
StaticSlot g_static[STATIC_MAX_DEVICES];
std::mutex g_static_lock;                      // claiming and releasing a slot
}  // namespace

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

// First launch of a kernel by this context: raise its dynamic-LDS limit, and check that a workgroup fits on a
// compute unit at all.  The forward is an ordinary launch of one workgroup per compute unit whose grid barriers need
// all of them resident at once; a kernel that cannot be resident is refused here instead of running into the
// bounded wait.  (Another process that holds compute units can still make a launch time out.)
template <class Kern>
int ensure_lds(sd_ctx* c, Kern kern, size_t bytes) {
    const void* key = reinterpret_cast<const void*>(kern);
    for (int i = 0; i < c->n_lds_done; ++i)
        if (c->lds_done[i] == key) return SD_OK;
    if (bytes > 48 * 1024) HIPCHK(c, hipFuncSetAttribute(key, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    int resident = 0;
    HIPCHK(c, hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, key, WG_THREADS, bytes));
    if (resident < 1) return SD_EINVAL;
    if (c->n_lds_done < LDS_DONE_MAX) c->lds_done[c->n_lds_done++] = key;
    return SD_OK;
}

// The tiled copy of the layer matrices: per layer QKV, O, gate/up, down, each as large as its matrices.
struct TiledLayout { size_t qkv, o, gateup, down, per_layer; };
TiledLayout tiled_layout(const sd_config& g) {
    const size_t d = g.d_model, hq = (size_t)g.n_heads * g.head_dim, hkv = (size_t)g.n_kv_heads * g.head_dim, F = g.d_ffn;
    TiledLayout t;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    t.qkv = take((hq + 2 * hkv) * d * 2); t.o = take(d * hq * 2); t.gateup = take(2 * F * d * 2); t.down = take(d * F * 2);
    t.per_layer = off;
    return t;
}
// the grid of the forward kernels on the current device (one workgroup per compute unit)
int forward_grid() {
    int dev = 0, n = 256;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        n = prop.multiProcessorCount;
    else
        (void)hipGetLastError();
    return n > HEAD_GRID_MAX ? HEAD_GRID_MAX : n;
}

// The phase list of one forward: embedding, then for every layer the sub-layers that are not skipped, then
// the output head.  A skipped sub-layer contributes nothing and writes no keys / values (Alg. 1: the draft is
// the target minus the prune set); the residual stream simply passes to the next phase that runs.
std::vector<Phase> build_program(const sd_ctx* c, bool use_skip) {
    const sd_config& g = c->cfg;
    const Carve& cv = c->cv;
    const size_t esz = esize(&g);
    const size_t plane = (size_t)g.n_kv_heads * g.max_seq * g.head_dim * esz;   // bytes per K or V plane
    const int hq = g.n_heads * g.head_dim, hkv = g.n_kv_heads * g.head_dim;
    // The decode-time kernels read the O and down projections from the tiled copy (sd_set_tiled_weights) when every
    // workgroup's rows are whole 16-row tiles of the copy's numbering: the down projection's stream runs 15 % faster for
    // it (measured per phase on the 7B shape: down 21.0 -> 18.9 us per layer; O 10.3 -> 9.6).  Not QKV, whose tiles
    // would fit as well: its stream gains 0.3 us and the grid barrier behind it loses 1 us to a wider spread between
    // workgroups.  Not gate/up: its units do not divide into whole tiles per workgroup, and a copy cut by workgroup
    // (tried) gained nothing there -- short rows, 8 + 8 of them per tile.
    const TiledLayout tl = tiled_layout(g);
    auto tiled_at = [&](int l, size_t off, bool whole) -> const void* {
        return (c->tiled && whole) ? c->tiled + (size_t)l * tl.per_layer + off : nullptr;
    };
    const bool rows_whole = c->n_cu > 0 && g.d_model % (16 * c->n_cu) == 0;
    std::vector<Phase> prog;
    auto blank = [](int kind, int layer) { Phase p; std::memset(&p, 0, sizeof(p)); p.kind = kind; p.layer = layer; return p; };
    char* acts = c->ws + cv.acts;
    float* h = reinterpret_cast<float*>(acts);
    {
        Phase p = blank(PK_EMBED, -1);
        p.out = h;
        prog.push_back(p);
    }
    const size_t per_layer = 2 * cv.act_q + 2 * cv.act_h + cv.act_a;
    for (int l = 0; l < g.n_layers; ++l) {
        const LayerPtrs& lp = c->layers[l];
        const int sk = use_skip ? c->skip[l] : 0;
        char* base = acts + cv.act_h + (size_t)l * per_layer;
        float* q = reinterpret_cast<float*>(base);
        float* att = reinterpret_cast<float*>(base + cv.act_q);
        float* h1 = reinterpret_cast<float*>(base + 2 * cv.act_q);
        float* a = reinterpret_cast<float*>(base + 2 * cv.act_q + cv.act_h);
        float* h2 = reinterpret_cast<float*>(base + 2 * cv.act_q + cv.act_h + cv.act_a);
        char* kc = c->kv + (size_t)(2 * l) * plane;
        char* vc = kc + plane;
        if (!(sk & SD_SKIP_ATTN)) {
            Phase p = blank(PK_QKV, l);
            p.Kd = g.d_model; p.N = hq + 2 * hkv; p.n_units = p.N / 16;
            p.w[0] = lp.wq; p.w[1] = lp.wk; p.w[2] = lp.wv; p.gain = lp.attn_norm; p.xin = h; p.out = q; p.kc = kc; p.vc = vc;
            p.wt = tiled_at(l, tl.qkv, false);
            prog.push_back(p);
            p = blank(PK_ATTN, l);
            p.N = hq; p.xin = q; p.out = att; p.kc = kc; p.vc = vc;
            prog.push_back(p);
            p = blank(PK_OPROJ, l);
            p.Kd = hq; p.N = g.d_model; p.n_units = p.N;
            p.w[0] = lp.wo; p.xin = att; p.res = h; p.out = h1;
            p.wt = tiled_at(l, tl.o, rows_whole);
            prog.push_back(p);
            h = h1;
        }
        if (!(sk & SD_SKIP_FFN)) {
            Phase p = blank(PK_GATEUP, l);
            p.Kd = g.d_model; p.N = g.d_ffn; p.n_units = p.N;
            p.w[0] = lp.wg; p.w[1] = lp.wu; p.gain = lp.ffn_norm; p.xin = h; p.out = a;
            prog.push_back(p);
            p = blank(PK_DOWN, l);
            p.Kd = g.d_ffn; p.N = g.d_model; p.n_units = p.N;
            p.w[0] = lp.wd; p.xin = a; p.res = h; p.out = h2;
            p.wt = tiled_at(l, tl.down, rows_whole);
            prog.push_back(p);
            h = h2;
        }
    }
    {
        Phase p = blank(PK_HEAD, -1);
        p.Kd = g.d_model; p.N = g.vocab; p.n_units = p.N;
        p.w[0] = c->lm_head; p.gain = c->final_norm; p.xin = h;
        prog.push_back(p);
    }
    prog.push_back(blank(PK_END, -1));
    return prog;
}

int upload_program(sd_ctx* c, bool draft) {
    std::vector<Phase> prog = build_program(c, draft);
    c->n_prog[draft ? 1 : 0] = (int)prog.size();
    HIPCHK(c, hipMemcpyAsync(c->ws + (draft ? c->cv.prog_draft : c->cv.prog_target), prog.data(),
                             prog.size() * sizeof(Phase), hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));   // the host vector goes out of scope
    return SD_OK;
}

// the output head alone: final norm and output projection of the row at the start of the activation region (where the
// matrix-matrix prompt path leaves the prompt's last residual row)
int upload_head_program(sd_ctx* c) {
    const sd_config& g = c->cfg;
    Phase prog[2];
    std::memset(prog, 0, sizeof(prog));
    prog[0].kind = PK_HEAD; prog[0].layer = -1;
    prog[0].Kd = g.d_model; prog[0].N = g.vocab; prog[0].n_units = g.vocab;
    prog[0].w[0] = c->lm_head; prog[0].gain = c->final_norm;
    prog[0].xin = reinterpret_cast<const float*>(c->ws + c->cv.acts + c->panel.h_last);
    prog[1].kind = PK_END; prog[1].layer = -1;
    HIPCHK(c, hipMemcpyAsync(c->ws + c->cv.prog_head, prog, sizeof(prog), hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));   // the host array goes out of scope
    return SD_OK;
}

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
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, c->stream, reinterpret_cast<unsigned*>(c->ws + c->cv.bar), BAR_WORDS);
    // the diagnostics' records start empty whatever the workspace held before
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, c->stream,
                       reinterpret_cast<unsigned*>(c->ws + c->cv.trace + sizeof(unsigned long long) * TRACE_CAP), 2);
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, c->stream, reinterpret_cast<unsigned*>(c->ws + c->cv.guard_rec), 64);
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipStreamSynchronize(c->stream));   // host vectors go out of scope
    c->n_cu = forward_grid();
    int e;
    if ((e = upload_program(c, false))) return e;   // (the phase lists depend on the grid size: see build_program)
    if ((e = upload_program(c, true))) return e;
    if ((e = upload_head_program(c))) return e;
    c->span = c->span_mode < 0 ? span_pays(&c->cfg, c->n_cu) : c->span_mode != 0;
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

// one forward = one launch of the persistent kernel, one workgroup per compute unit
enum { PROG_TARGET = 0, PROG_DRAFT = 1, PROG_HEAD = 2 };   // which phase list a forward walks

template <typename WT>
int forward(sd_ctx* c, Rows rows, int which, HeadPlan hp) {
    const sd_config& g = c->cfg;
    FwdArgs A;
    std::memset(&A, 0, sizeof(A));
    A.prog = reinterpret_cast<const Phase*>(c->ws + (which == PROG_DRAFT ? c->cv.prog_draft
                                                  : which == PROG_HEAD ? c->cv.prog_head : c->cv.prog_target));
    A.L = LayerDims{g.d_model, g.n_heads, g.n_kv_heads, g.head_dim, g.d_ffn, g.vocab, g.max_seq};
    A.rows = rows;
    A.st = c->st();
    A.prompt = c->prompt();
    A.tok_emb = c->tok_emb;
    A.cosT = c->f(c->cv.cosT); A.sinT = c->f(c->cv.sinT);
    A.part_o = c->f(c->cv.part_o); A.part_ml = c->f(c->cv.part_ml);
    A.att_counters = reinterpret_cast<unsigned*>(c->ws + c->cv.counters);
    A.head.logits = hp.logits;
    A.head.part_val = c->f(c->cv.head_val);
    A.head.part_idx = reinterpret_cast<int*>(c->ws + c->cv.head_idx);
    A.head.dst = hp.dst; A.head.off = hp.off;
    A.head_run = hp.run ? 1 : 0;
    A.head_row_from = hp.run ? hp.row_from : 0;
    {
        const int hq = g.n_heads * g.head_dim, hkv = g.n_kv_heads * g.head_dim;
        A.kind_units[PK_QKV] = (hq + 2 * hkv) / 16; A.kind_Kd[PK_QKV] = g.d_model;
        A.kind_units[PK_OPROJ] = g.d_model; A.kind_Kd[PK_OPROJ] = hq;
        A.kind_units[PK_GATEUP] = g.d_ffn; A.kind_Kd[PK_GATEUP] = g.d_model;
        A.kind_units[PK_DOWN] = g.d_model; A.kind_Kd[PK_DOWN] = g.d_ffn;
        A.kind_units[PK_HEAD] = g.vocab; A.kind_Kd[PK_HEAD] = g.d_model;
    }
    A.eps = g.rms_eps;
    A.bar = reinterpret_cast<unsigned*>(c->ws + c->cv.bar);
    A.spin_limit = c->spin_limit;
    A.n_prog = which == PROG_HEAD ? 2 : c->n_prog[which == PROG_DRAFT ? 1 : 0];
    A.trace = c->trace_on ? reinterpret_cast<unsigned long long*>(c->ws + c->cv.trace) : nullptr;
    A.trace_cap = TRACE_CAP;
#ifdef SDFP_WAVETRACE
    if (A.trace) HIPCHK(c, hipMemsetAsync(A.trace, 0, sizeof(unsigned long long) * (TRACE_CAP + 1), c->stream));
#endif
    A.guard.lo[0] = c->ws; A.guard.hi[0] = c->ws + c->cv.total;
    A.guard.lo[1] = c->kv; A.guard.hi[1] = c->kv + sd_kv_bytes(&c->cfg);
    A.guard.lo[2] = c->w_lo; A.guard.hi[2] = c->w_hi;
    A.guard.rec = c->dbg_host ? c->dbg_host : reinterpret_cast<unsigned long long*>(c->ws + c->cv.guard_rec);
    A.guard.beacon = c->dbg_host ? reinterpret_cast<unsigned*>(c->dbg_host + 32) : nullptr;
    A.guard.probe = c->dbg_host ? c->dbg_host + 32 + HEAD_GRID_MAX * 8 : nullptr;   // after 1024*8*2 beacons
    A.guard.prog = A.prog;
    A.guard.prog_len = (int)prog_len(&c->cfg);
    if (rows.M < 1 || rows.M > MAX_ROWS) return SD_EINVAL;
    const size_t lds = LDS_DYN_BYTES;
    static_assert(attn_lds_bytes(128, MAX_ROWS * 8) <= (size_t)LDS_ZERO_OFF, "attention LDS must fit");
    int e;
    auto launch = [&](auto kern) -> int {
        if ((e = ensure_lds(c, kern, lds))) return e;
        hipLaunchKernelGGL(kern, dim3(c->n_cu), dim3(WG_THREADS), lds, c->stream, A);
        HIPCHK(c, hipGetLastError());
        return SD_OK;
    };
    const int role = rows.src == ROWS_PROMPT ? 0 : (rows.src == ROWS_DRAFT ? 1 : (rows.M == 1 ? 3 : 2));
    // outside prompt chunks the rows are handed over by data, and the row that readers poll is row 0 of a buffer:
    // the output head must start at row 0 there (it does: draft, verify and plain decode take logits of every row)
    if (role != 0 && hp.run && hp.row_from != 0) return SD_EINVAL;
    // contexts of more than 8 attention splits are possible: the instances that hold the merge of many splits
    const bool long_ctx = n_splits(&c->cfg) > 8;
#define SDFP_LAUNCH_ROWS(LPP, SPAN, LC)                                   \
    switch (role) {                                                      \
        case 1: return launch(k_forward<WT, 1, LPP, 1, SPAN, LC>);         \
        case 3: return launch(k_forward<WT, 3, LPP, 1, SPAN, LC>);         \
        default:                                                         \
            switch (rows.M) {                                            \
                case 2: return launch(k_forward<WT, 2, LPP, 2, SPAN, LC>); \
                case 3: return launch(k_forward<WT, 2, LPP, 3, SPAN, LC>); \
                case 4: return launch(k_forward<WT, 2, LPP, 4, SPAN, LC>); \
                case 5: return launch(k_forward<WT, 2, LPP, 5, SPAN, LC>); \
                case 6: return launch(k_forward<WT, 2, LPP, 6, SPAN, LC>); \
                case 7: return launch(k_forward<WT, 2, LPP, 7, SPAN, LC>); \
                case 8: return launch(k_forward<WT, 2, LPP, 8, SPAN, LC>); \
                case 9: return launch(k_forward<WT, 2, LPP, 9, SPAN, LC>); \
                default: return SD_EINVAL;                               \
            }                                                            \
    }
#define SDFP_LAUNCH_HD(LPP)                                              \
    if (role == 0) return launch(k_forward<WT, 0, LPP, 0, false, true>);                 \
    if (long_ctx) {                                                                      \
        if (c->span) { SDFP_LAUNCH_ROWS(LPP, true, true) } else { SDFP_LAUNCH_ROWS(LPP, false, true) }   \
    } else {                                                                             \
        if (c->span) { SDFP_LAUNCH_ROWS(LPP, true, false) } else { SDFP_LAUNCH_ROWS(LPP, false, false) } \
    }
    switch (g.head_dim) {   // config_ok admits 16, 32, 64, 128
        case 16: SDFP_LAUNCH_HD(4)
        case 32: SDFP_LAUNCH_HD(8)
        case 64: SDFP_LAUNCH_HD(16)
        default: SDFP_LAUNCH_HD(32)
    }
#undef SDFP_LAUNCH_HD
#undef SDFP_LAUNCH_ROWS
}

// ---- the prompt as matrix-matrix products (sdfp_prefill.hip.h): panels of P rows, per layer a norm / split kernel,
// the QKV GEMM (rotary, cache rows, queries), attention in 16-row chunks, the O GEMM, norm / split, the gate/up GEMM
// (SwiGLU, pieces of its output) and the down GEMM; then the output head for the prompt's last row through the one-row
// forward kernel with a phase list that holds the head alone.
template <class Kern>
int launch_pf(sd_ctx* c, Kern kern, dim3 grid, dim3 block, size_t lds, const PfGemm& a) {
    int e = ensure_lds(c, kern, lds);
    if (e) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, c->stream, a);
    return SD_OK;
}
int launch_pf_attn(sd_ctx* c, const PfAttn& a, int n_wg) {
    const sd_config& g = c->cfg;
    const size_t lds = attn_lds_bytes(g.head_dim, MAX_ROWS * (g.n_heads / g.n_kv_heads), ATT_QC_PANEL, true);
    int e;
    const bool long_ctx = a.pos0 + a.M > 8 * ATT_SL;   // the panel's last row sees more than 8 splits
#define SDFP_PF_ATTN_1(LPP, LC)                                                                  \
    if ((e = ensure_lds(c, k_pf_attn<LPP, LC>, lds))) return e;                                  \
    hipLaunchKernelGGL((k_pf_attn<LPP, LC>), dim3(n_wg), dim3(WG_THREADS), lds, c->stream, a);    \
    return SD_OK;
#define SDFP_PF_ATTN(LPP) if (long_ctx) { SDFP_PF_ATTN_1(LPP, true) } else { SDFP_PF_ATTN_1(LPP, false) }
    switch (g.head_dim) {
        case 16: SDFP_PF_ATTN(4)
        case 32: SDFP_PF_ATTN(8)
        case 64: SDFP_PF_ATTN(16)
        default: SDFP_PF_ATTN(32)
    }
#undef SDFP_PF_ATTN
#undef SDFP_PF_ATTN_1
}

int do_prefill_gemm(sd_ctx* c, int n, HeadPlan hp) {
    const sd_config& g = c->cfg;
    const PanelPlan& pl = c->panel;
    const int d = g.d_model, hq = g.n_heads * g.head_dim, hkv = g.n_kv_heads * g.head_dim, F = g.d_ffn;
    const size_t plane = (size_t)g.n_kv_heads * g.max_seq * g.head_dim;   // elements per K or V plane
    char* base = c->ws + c->cv.acts;
    float* h = reinterpret_cast<float*>(base + pl.h);
    float* q = reinterpret_cast<float*>(base + pl.q);
    float* att = reinterpret_cast<float*>(base + pl.att);
    float* rs = reinterpret_cast<float*>(base + pl.rs);
    bf16_t* xs_a = reinterpret_cast<bf16_t*>(base + pl.xs_a);
    bf16_t* xs_b = reinterpret_cast<bf16_t*>(base + pl.xs_b);
    unsigned* counters = reinterpret_cast<unsigned*>(base + pl.counters);
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(256), 0, c->stream, counters, PANEL_MAX_AWG);
    const LayerDims L{g.d_model, g.n_heads, g.n_kv_heads, g.head_dim, g.d_ffn, g.vocab, g.max_seq};
    int e;
    float* shares = reinterpret_cast<float*>(base + pl.shares);
    // O / down projections have few outputs: deal a tile's shares to as many workgroups as it takes to fill the chip
    auto share_groups = [&](int n_nt, int my) {
        int gcount = 1;
        while (gcount < PF_NSHARE && n_nt * my * gcount < (c->n_cu * 3) / 4) gcount *= 2;
        return gcount;
    };
    auto gemm_grid = [](const PfGemm& a) { return dim3((unsigned)((a.n_nt * a.n_groups + 7) / 8 * 8 * a.my)); };
    const TiledLayout tl = tiled_layout(g);
    auto tiled_at = [&](int l, size_t off) {
        return c->tiled ? reinterpret_cast<const bf16_t*>(c->tiled + (size_t)l * tl.per_layer + off) : nullptr;
    };
    // weight tiles per wave: 3 (QKV, gate/up) or 4 (O, down) when the panel has rows enough to fill the chip with such
    // tiles, else 1 (a short prompt is bound by the read of the weights and wants many workgroups, not large tiles)
    constexpr int NT_WIDE = 3, NT_NARROW = 4;
    // (measured on the 7B shape: the one-tile kernels win only below about 3/8 of the compute units' worth of large
    // tiles -- they read as many LDS bytes per matrix-core step as they feed it)
    auto tiles_fill = [&](int n_tiles, int nt, int my, int groups) {
        return ((n_tiles + 8 * nt - 1) / (8 * nt)) * my * groups >= (c->n_cu * 3) / 8;
    };
    // QKV and gate/up: 1, 2 or 3 tiles per wave -- whichever needs the least time by a simple model: rounds of workgroups
    // on the compute units x tiles per wave x the relative cost of a tile at that size (smaller workgroup tiles read
    // more LDS and L2 bytes per matrix-core instruction).  290 workgroups of 3 tiles are two rounds, 430 of 2 tiles two
    // cheaper ones; 116 of 3 tiles fill half the chip, 172 of 2 tiles two thirds of it in two thirds of the time.
    auto pick_nt = [&](int n_tiles, int my) {
        const double w[4] = {0.0, 1.4, 1.1, 1.0};
        int best = 3;
        double best_cost = 1e30;
        for (int nt = 3; nt >= 1; --nt) {
            const int wgs = ((n_tiles + 8 * nt - 1) / (8 * nt)) * my;
            const double cost = (double)((wgs + c->n_cu - 1) / c->n_cu) * nt * w[nt];
            if (cost < best_cost - 1e-9) { best_cost = cost; best = nt; }
        }
        return best;
    };
    for (int p0 = 0; p0 < n; p0 += pl.P) {
        const int np = std::min(pl.P, n - p0);
        const dim3 blk(WG_THREADS);
        // the share sums of a projection of `outs` outputs fit the scratch that is sized for the panel's O / down sums
        auto dealt_fits = [&](int outs) { return (size_t)np * outs <= (size_t)pl.P * d; };
        // the one-tile kernels multiply only the 16-row column tiles a short panel has
        const int jt = np <= 16 ? 1 : (np <= 32 ? 2 : 4);
#define SDFP_PF_ONE_TILE(KIND, PART)                                                                               \
    (jt == 1 ? launch_pf(c, k_pf_gemm<KIND, 1, PART, 1>, gemm_grid(a), blk, PF_LDS_BYTES, a)                      \
             : jt == 2 ? launch_pf(c, k_pf_gemm<KIND, 1, PART, 2>, gemm_grid(a), blk, PF_LDS_BYTES, a)            \
                       : launch_pf(c, k_pf_gemm<KIND, 1, PART, 4>, gemm_grid(a), blk, PF_LDS_BYTES, a))
        const int my = (np + PF_TM - 1) / PF_TM;
        const bool fused = d <= PF_FUSED_MAX_D;   // residual + row norm + split in one kernel (rows that fit its registers)
        hipLaunchKernelGGL(k_pf_embed, dim3(np), dim3(256), 0, c->stream, c->prompt() + p0,
                           reinterpret_cast<const bf16_t*>(c->tok_emb), d, g.vocab, h);
        for (int l = 0; l < g.n_layers; ++l) {
            const LayerPtrs& lp = c->layers[l];
            bf16_t* kc = reinterpret_cast<bf16_t*>(c->kv) + (size_t)(2 * l) * plane;
            bf16_t* vc = kc + plane;
            PfGemm a;
            std::memset(&a, 0, sizeof(a));
            a.M = np; a.pos0 = p0; a.L = L; a.cosT = c->f(c->cv.cosT); a.sinT = c->f(c->cv.sinT);
            a.my = my; a.part = shares; a.part_arr = (size_t)np * d; a.part_ld = d;
            // attention sub-layer (with the residual update that the previous layer's down projection left to do)
            if (fused) {
                hipLaunchKernelGGL(k_pf_residual_norm_split, dim3(np), dim3(WG_THREADS), 0, c->stream, h,
                                   l > 0 ? (const float*)shares : (const float*)nullptr, (size_t)np * d, d, g.rms_eps,
                                   lp.attn_norm, rs, xs_a, pf_xs_piece(np, d));
            } else {
                hipLaunchKernelGGL(k_pf_rownorm, dim3(np), dim3(WG_THREADS), 0, c->stream, h, d, g.rms_eps, rs);
                hipLaunchKernelGGL(k_pf_split, dim3(1024), dim3(256), 0, c->stream, h, lp.attn_norm, np, d, xs_a, pf_xs_piece(np, d));
            }
            a.w[0] = (const bf16_t*)lp.wq; a.w[1] = (const bf16_t*)lp.wk; a.w[2] = (const bf16_t*)lp.wv;
            a.xs = xs_a; a.xs_piece = pf_xs_piece(np, d); a.Kd = d; a.n_tiles = (hq + 2 * hkv) / 16; a.rs = rs;
            a.wt = tiled_at(l, tl.qkv);
            a.q = q; a.kc = kc; a.vc = vc;
            a.n_groups = 1;
            const int nt_qkv = pick_nt(a.n_tiles, my);
            if (nt_qkv > 1) {
                a.n_nt = (a.n_tiles + 8 * nt_qkv - 1) / (8 * nt_qkv);
                e = nt_qkv == 3 ? launch_pf(c, k_pf_gemm<PF_QKV, 3, false>, gemm_grid(a), blk, PF_LDS_BYTES, a)
                                : launch_pf(c, k_pf_gemm<PF_QKV, 2, false>, gemm_grid(a), blk, PF_LDS_BYTES, a);
            } else if (dealt_fits(a.n_tiles * 16) && share_groups((a.n_tiles + 7) / 8, my) > 1) {
                // short prompt: shares dealt to workgroups, then the epilogue
                a.n_nt = (a.n_tiles + 7) / 8; a.n_groups = share_groups(a.n_nt, my);
                a.part_ld = a.n_tiles * 16; a.part_arr = (size_t)np * a.part_ld;
                e = SDFP_PF_ONE_TILE(PF_QKV, true);
                hipLaunchKernelGGL(k_pf_finish_qkv, dim3(512), dim3(256), 0, c->stream, a);
                a.part_ld = d; a.part_arr = (size_t)np * d;
            } else {
                a.n_nt = (a.n_tiles + 7) / 8;
                e = SDFP_PF_ONE_TILE(PF_QKV, false);
            }
            if (e) return e;
            PfAttn t;
            std::memset(&t, 0, sizeof(t));
            t.q = q; t.att = att; t.kc = kc; t.vc = vc;
            t.part = reinterpret_cast<float*>(base + pl.part); t.part_stride = pl.part_stride; t.part_ml_off = pl.part_ml_off;
            t.counters = counters; t.M = np; t.pos0 = p0; t.L = L;
            const int items = ((np + MAX_ROWS - 1) / MAX_ROWS) * g.n_kv_heads;
            if ((e = launch_pf_attn(c, t, std::min(pl.n_awg, items)))) return e;
            hipLaunchKernelGGL(k_pf_split, dim3(1024), dim3(256), 0, c->stream, att, (const float*)nullptr, np, hq, xs_a, pf_xs_piece(np, hq));
            a.w[0] = (const bf16_t*)lp.wo; a.w[1] = a.w[2] = nullptr;
            a.xs = xs_a; a.xs_piece = pf_xs_piece(np, hq); a.Kd = hq; a.n_tiles = d / 16; a.rs = nullptr; a.h = h;
            a.wt = tiled_at(l, tl.o);
            if (tiles_fill(a.n_tiles, NT_NARROW, my, PF_NSHARE)) {
                a.n_nt = (a.n_tiles + 8 * NT_NARROW - 1) / (8 * NT_NARROW); a.n_groups = share_groups(a.n_nt, my);
                e = launch_pf(c, k_pf_gemm<PF_OPROJ, NT_NARROW, true>, gemm_grid(a), blk, PF_LDS_BYTES, a);
            } else {
                a.n_nt = (a.n_tiles + 7) / 8; a.n_groups = share_groups(a.n_nt, my);
                e = SDFP_PF_ONE_TILE(PF_OPROJ, true);
            }
            if (e) return e;
            // feed-forward sub-layer
            if (fused) {
                hipLaunchKernelGGL(k_pf_residual_norm_split, dim3(np), dim3(WG_THREADS), 0, c->stream, h, (const float*)shares,
                                   a.part_arr, d, g.rms_eps, lp.ffn_norm, rs, xs_a, pf_xs_piece(np, d));
            } else {
                hipLaunchKernelGGL(k_pf_residual, dim3(512), dim3(256), 0, c->stream, h, shares, a.part_arr, np * d / 4);
                hipLaunchKernelGGL(k_pf_rownorm, dim3(np), dim3(WG_THREADS), 0, c->stream, h, d, g.rms_eps, rs);
                hipLaunchKernelGGL(k_pf_split, dim3(1024), dim3(256), 0, c->stream, h, lp.ffn_norm, np, d, xs_a, pf_xs_piece(np, d));
            }
            a.w[0] = (const bf16_t*)lp.wg; a.w[1] = (const bf16_t*)lp.wu;
            a.xs = xs_a; a.xs_piece = pf_xs_piece(np, d); a.Kd = d; a.n_tiles = F / 8; a.rs = rs;
            a.wt = tiled_at(l, tl.gateup);
            a.xs_out = xs_b; a.xs_out_piece = pf_xs_piece(np, F);
            a.n_groups = 1;
            const int nt_gu = pick_nt(a.n_tiles, my);
            if (nt_gu > 1) {
                a.n_nt = (a.n_tiles + 8 * nt_gu - 1) / (8 * nt_gu);
                e = nt_gu == 3 ? launch_pf(c, k_pf_gemm<PF_GATEUP, 3, false>, gemm_grid(a), blk, PF_LDS_BYTES, a)
                               : launch_pf(c, k_pf_gemm<PF_GATEUP, 2, false>, gemm_grid(a), blk, PF_LDS_BYTES, a);
            } else {   // (dealing the shares as for QKV does not pay here: 172 workgroups as it is, 72 vs 65 us on the 7B shape)
                a.n_nt = (a.n_tiles + 7) / 8;
                e = SDFP_PF_ONE_TILE(PF_GATEUP, false);
            }
            if (e) return e;
            a.w[0] = (const bf16_t*)lp.wd; a.w[1] = nullptr;
            a.xs = xs_b; a.xs_piece = pf_xs_piece(np, F); a.Kd = F; a.n_tiles = d / 16; a.rs = nullptr;
            a.wt = tiled_at(l, tl.down);
            if (tiles_fill(a.n_tiles, NT_NARROW, my, PF_NSHARE)) {
                a.n_nt = (a.n_tiles + 8 * NT_NARROW - 1) / (8 * NT_NARROW); a.n_groups = share_groups(a.n_nt, my);
                e = launch_pf(c, k_pf_gemm<PF_DOWN, NT_NARROW, true>, gemm_grid(a), blk, PF_LDS_BYTES, a);
            } else {
                a.n_nt = (a.n_tiles + 7) / 8; a.n_groups = share_groups(a.n_nt, my);
                e = SDFP_PF_ONE_TILE(PF_DOWN, true);
            }
            if (e) return e;
            // the down projection's residual update: fused into the next layer's first kernel, or done here
            if (!fused || l == g.n_layers - 1)
                hipLaunchKernelGGL(k_pf_residual, dim3(512), dim3(256), 0, c->stream, h, shares, a.part_arr, np * d / 4);
        }
#undef SDFP_PF_ONE_TILE
        if (p0 + pl.P >= n)   // the prompt's last row goes to the output head
            HIPCHK(c, hipMemcpyAsync(base + pl.h_last, h + (size_t)(np - 1) * d, (size_t)d * 4, hipMemcpyDeviceToDevice, c->stream));
    }
    HIPCHK(c, hipGetLastError());
    return forward<bf16_t>(c, Rows{1, ROWS_VERIFY, 0}, PROG_HEAD, hp);
}

template <typename WT>
int do_prefill(sd_ctx* c, const int32_t* prompt_host, int n, int mode, const float* u_host) {
    int e = lazy_device_init(c);
    if (e) return e;
    HIPCHK(c, hipMemcpyAsync(c->prompt(), prompt_host, sizeof(int) * (size_t)n, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));   // prompt_host may be reused by the caller on return
    // a fresh sequence starts from clean barrier and split-merge counters (also the way out of SD_ETIMEOUT)
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, c->stream, reinterpret_cast<unsigned*>(c->ws + c->cv.bar), BAR_WORDS);
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, c->stream, reinterpret_cast<unsigned*>(c->ws + c->cv.counters),
                       c->cfg.n_kv_heads);
    const bool keep = mode == SD_SAMPLE || c->keep_logits;
    const bool gemm = std::is_same<WT, bf16_t>::value && c->panel.P > 0 &&
                      (c->prefill_mode == 1 || (c->prefill_mode < 0 && n >= PREFILL_MATRIX_MIN_ROWS));
    if (gemm) {
        HeadPlan hp{true, 0, keep ? c->f(c->cv.zp) : nullptr, ROWS_VERIFY, 0};
        if ((e = do_prefill_gemm(c, n, hp))) return e;
    } else {
        for (int p0 = 0; p0 < n; p0 += PREFILL_ROWS) {
            Rows rows{std::min(PREFILL_ROWS, n - p0), ROWS_PROMPT, p0};
            const bool last = p0 + PREFILL_ROWS >= n;
            HeadPlan hp{last, rows.M - 1, c->f(c->cv.zp), ROWS_VERIFY, 0};
            if (last && !keep) hp.logits = nullptr;
            if ((e = forward<WT>(c, rows, PROG_TARGET, hp))) return e;
        }
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
        int e = forward<WT>(c, rows, PROG_DRAFT, hp);
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
    return forward<WT>(c, rows, PROG_TARGET, hp);
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

// the argument checks of context creation that do not concern the workspace
int check_init_args(const sd_config* cfg, const sd_weights* w, const void* kv_buf, size_t kv_bytes) {
    if (!config_ok(cfg) || !w || !kv_buf) return SD_EINVAL;
    if ((uintptr_t)kv_buf & 255) return SD_EINVAL;
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
    if (kv_bytes < align_up((size_t)cfg->n_layers * 2 * cfg->n_kv_heads * cfg->max_seq * cfg->head_dim * esize(cfg)))
        return SD_ENOMEM;
    return SD_OK;
}

// fill a context whose arguments have been checked; layers / skip: storage for n_layers entries each
void fill_ctx(sd_ctx* c, LayerPtrs* layers, uint8_t* skip, const sd_config* cfg, const sd_weights* w,
              const uint8_t* skip_mask, void* kv_buf, void* ws_buf, void* hip_stream, bool compact = false) {
    c->cfg = *cfg;
    c->layers = layers;
    c->skip = skip;
    for (int l = 0; l < cfg->n_layers; ++l) {
        c->layers[l] = LayerPtrs{w->attn_norm[l], w->ffn_norm[l], w->wq[l], w->wk[l], w->wv[l],
                                 w->wo[l], w->w_gate[l], w->w_up[l], w->w_down[l]};
        c->skip[l] = skip_mask ? (uint8_t)(skip_mask[l] & 3) : (uint8_t)0;
    }
    c->tok_emb = w->tok_emb; c->lm_head = w->lm_head; c->final_norm = w->final_norm;
    c->kv = (char*)kv_buf; c->ws = (char*)ws_buf;
    c->stream = (hipStream_t)hip_stream;
    c->cv = carve(cfg, compact);
    c->phase = PH_INIT;
    c->dev_ready = false; c->keep_logits = false;
    c->hip_err = 0; c->P_hi = 0; c->out_hi = 0; c->K_cur = 0; c->mode_cur = SD_GREEDY; c->n_cu = 256;
    c->spin_limit = 1u << 21; c->trace_on = false; c->span = false; c->span_mode = -1;
    c->n_lds_done = 0;
    c->static_dev = -1;
    c->prefill_mode = -1;
    c->tiled = nullptr;
    c->panel = plan_panel(cfg, c->cv.acts_bytes);
    const size_t es = esize(cfg), d = (size_t)cfg->d_model, hq = (size_t)cfg->n_heads * cfg->head_dim,
                 hkv = (size_t)cfg->n_kv_heads * cfg->head_dim, F = (size_t)cfg->d_ffn, V = (size_t)cfg->vocab;
    const char *lo = (const char*)w->tok_emb, *hi = lo;
    auto span = [&](const void* p, size_t bytes) {
        const char* q = (const char*)p;
        if (q < lo) lo = q;
        if (q + bytes > hi) hi = q + bytes;
    };
    span(w->tok_emb, V * d * es); span(w->lm_head, V * d * es); span(w->final_norm, d * 4);
    for (int l = 0; l < cfg->n_layers; ++l) {
        span(w->attn_norm[l], d * 4); span(w->ffn_norm[l], d * 4);
        span(w->wq[l], hq * d * es); span(w->wk[l], hkv * d * es); span(w->wv[l], hkv * d * es);
        span(w->wo[l], d * hq * es); span(w->w_gate[l], F * d * es); span(w->w_up[l], F * d * es);
        span(w->w_down[l], d * F * es);
    }
    c->w_lo = lo; c->w_hi = hi;
    c->dbg_host = nullptr;
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
    if (!ws_buf || ((uintptr_t)ws_buf & 255)) return SD_EINVAL;
    int e = check_init_args(cfg, w, kv_buf, kv_bytes);
    if (e) return e;
    if (ws_bytes < sd_workspace_bytes(cfg)) return SD_ENOMEM;
    sd_ctx* c = new (std::nothrow) sd_ctx();
    LayerPtrs* layers = new (std::nothrow) LayerPtrs[cfg->n_layers];
    uint8_t* skip = new (std::nothrow) uint8_t[cfg->n_layers];
    if (!c || !layers || !skip) {
        delete c; delete[] layers; delete[] skip;
        return SD_ENOMEM;
    }
    fill_ctx(c, layers, skip, cfg, w, skip_mask, kv_buf, ws_buf, hip_stream);
    *out = c;
    return SD_OK;
}

int sd_init_static(sd_ctx** out, const sd_config* cfg, const sd_weights* w, const uint8_t* skip_mask, void* kv_buf,
                   size_t kv_bytes, void* hip_stream) {
    if (!out) return SD_EINVAL;
    *out = nullptr;
    int e = check_init_args(cfg, w, kv_buf, kv_bytes);
    if (e) return e;
    // the compact layout: the prompt path gets the room the decode kernels' buffers leave, not a full panel
    if (carve(cfg, true).total > (size_t)SD_STATIC_WS_BYTES || cfg->n_layers > SD_STATIC_MAX_LAYERS) return SD_ENOMEM;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return SD_EHIP;
    StaticSlot& slot = g_static[dev];
    std::lock_guard<std::mutex> claim(g_static_lock);
    if (slot.in_use) return SD_ESTATE;   // one context at a time shares the device's array
    if (!slot.ws) {                      // first call on this device, with the device current: where its copy lives
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SD_EHIP;
        slot.ws = p;
    }
    fill_ctx(&slot.ctx, slot.layers, slot.skip, cfg, w, skip_mask, kv_buf, slot.ws, hip_stream, true);
    slot.ctx.static_dev = dev;
    slot.in_use = true;
    *out = &slot.ctx;
    return SD_OK;
}

int sd_set_skip_mask(sd_ctx* c, const uint8_t* skip_mask) {
    if (!c || !skip_mask) return SD_EINVAL;
    if (c->phase == PH_DRAFTED) return SD_ESTATE;   // a drafted block must be verified with the mask it used
    for (int l = 0; l < c->cfg.n_layers; ++l) c->skip[l] = skip_mask[l] & 3;
    if (c->dev_ready) {
        HIPCHK(c, hipStreamSynchronize(c->stream));   // no enqueued draft forward reads the old list any more
        return upload_program(c, true);
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

int sd_set_spin_limit(sd_ctx* c, uint32_t polls) {
    if (!c || polls == 0) return SD_EINVAL;
    c->spin_limit = polls;
    return SD_OK;
}

int sd_set_turn_span(sd_ctx* c, int mode) {
    if (!c || mode < -1 || mode > 1) return SD_EINVAL;
    c->span_mode = mode;
    if (c->dev_ready) c->span = mode < 0 ? span_pays(&c->cfg, c->n_cu) : mode != 0;
    return SD_OK;
}

size_t sd_tiled_weights_bytes(const sd_config* cfg) {
    if (!cfg || cfg->dtype != SD_BF16 || !config_ok(cfg)) return 0;
    return tiled_layout(*cfg).per_layer * (size_t)cfg->n_layers;
}

int sd_set_tiled_weights(sd_ctx* c, void* buf, size_t bytes) {
    if (!c) return SD_EINVAL;
    auto reupload = [&]() -> int {   // the phase lists name the copy
        if (!c->dev_ready) return SD_OK;
        int e = upload_program(c, false);
        return e ? e : upload_program(c, true);
    };
    if (!buf) { c->tiled = nullptr; return reupload(); }
    const size_t need = sd_tiled_weights_bytes(&c->cfg);
    if (need == 0 || ((uintptr_t)buf & 255)) return SD_EINVAL;
    if (bytes < need) return SD_ENOMEM;
    const sd_config& g = c->cfg;
    const int d = g.d_model, hq = g.n_heads * g.head_dim, hkv = g.n_kv_heads * g.head_dim, F = g.d_ffn;
    c->n_cu = forward_grid();   // (the phase lists depend on it: see build_program)
    const TiledLayout tl = tiled_layout(g);
    PfGemm a;
    std::memset(&a, 0, sizeof(a));
    a.L = LayerDims{g.d_model, g.n_heads, g.n_kv_heads, g.head_dim, g.d_ffn, g.vocab, g.max_seq};
    const dim3 grid(2048), blk(256);
    for (int l = 0; l < g.n_layers; ++l) {
        const LayerPtrs& lp = c->layers[l];
        char* base = (char*)buf + (size_t)l * tl.per_layer;
        a.w[0] = (const bf16_t*)lp.wq; a.w[1] = (const bf16_t*)lp.wk; a.w[2] = (const bf16_t*)lp.wv;
        a.Kd = d; a.n_tiles = (hq + 2 * hkv) / 16;
        hipLaunchKernelGGL(k_pf_tile_weights<PF_QKV>, grid, blk, 0, c->stream, a, reinterpret_cast<bf16_t*>(base + tl.qkv));
        a.w[0] = (const bf16_t*)lp.wo; a.w[1] = a.w[2] = nullptr; a.Kd = hq; a.n_tiles = d / 16;
        hipLaunchKernelGGL(k_pf_tile_weights<PF_OPROJ>, grid, blk, 0, c->stream, a, reinterpret_cast<bf16_t*>(base + tl.o));
        a.w[0] = (const bf16_t*)lp.wg; a.w[1] = (const bf16_t*)lp.wu; a.Kd = d; a.n_tiles = F / 8;
        hipLaunchKernelGGL(k_pf_tile_weights<PF_GATEUP>, grid, blk, 0, c->stream, a, reinterpret_cast<bf16_t*>(base + tl.gateup));
        a.w[0] = (const bf16_t*)lp.wd; a.w[1] = nullptr; a.Kd = F; a.n_tiles = d / 16;
        hipLaunchKernelGGL(k_pf_tile_weights<PF_DOWN>, grid, blk, 0, c->stream, a, reinterpret_cast<bf16_t*>(base + tl.down));
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { c->hip_err = (int)e; return SD_EHIP; }
    c->tiled = (const char*)buf;
    return reupload();
}

int sd_set_prefill_mode(sd_ctx* c, int mode) {
    if (!c || mode < -1 || mode > 1) return SD_EINVAL;
    if (mode == 1 && c->panel.P <= 0) return SD_EINVAL;   // float32 storage, or no room for a panel in the workspace
    c->prefill_mode = mode;
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
#ifdef SDFP_WAVETRACE
    cnt = TRACE_CAP;
#endif
    if (cnt < 0 || cnt > TRACE_CAP) cnt = 0;
    *n = cnt;
    for (int i = 0; i < cnt && i < cap; ++i) host[i] = buf[i];
    return SD_OK;
}

int sd_guard_host_buffer(sd_ctx* c, uint64_t* pinned, size_t bytes) {
    if (!c) return SD_EINVAL;
    if (pinned && bytes < 32 * 8 + (size_t)HEAD_GRID_MAX * 8 * 2 * 4 + (size_t)HEAD_GRID_MAX * 8 * PROBE_N * 8) return SD_ENOMEM;
    c->dbg_host = reinterpret_cast<unsigned long long*>(pinned);
    return SD_OK;
}

int sd_guard_read(sd_ctx* c, uint64_t* host32) {
    if (!c || !host32) return SD_EINVAL;
    if (!c->dev_ready) return SD_ESTATE;
    HIPCHK(c, hipMemcpyAsync(host32, c->ws + c->cv.guard_rec, 32 * sizeof(uint64_t), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
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
    if (c->static_dev >= 0) {   // the static slot's context: nothing was allocated
        std::lock_guard<std::mutex> release(g_static_lock);
        g_static[c->static_dev].in_use = false;
        return;
    }
    delete[] c->layers;
    delete[] c->skip;
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

#include "sdfp_fit_host.hip.h"
