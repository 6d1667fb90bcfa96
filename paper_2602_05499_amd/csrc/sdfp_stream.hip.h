// Weight-streaming projections of the forward pass on the matrix cores, and their fused prologues / epilogues:
//   a2  RMSNorm -> QKV projection -> RoPE -> KV append
//   a4  O projection + residual           a6  down projection + residual
//   a5  RMSNorm -> gate/up projection -> SiLU * mul
//   a7  final RMSNorm -> output projection -> arg-max partials
//
// Shape of the work.  Y[m][n] = sum_k W[n][k] X[m][k] with M <= 16 activation rows: every weight is used once,
// so the phase is bound by the HBM read of W.  Output rows are grouped in TILES of 16 (the rows of one MFMA
// A operand); a workgroup owns a contiguous range of output rows and its 8 waves split the reduction dimension:
// a weight row is cut into BLOCKS of 2 KB, wave w takes the 4 consecutive 64-byte STEPS 4w..4w+3 of every block
// (two whole 128-byte lines of each of the 16 rows).  A step of a tile is one 16-byte load per lane -- lane l
// holds row l%16, bytes (l/16)*16.. of the step, which is exactly the A operand of v_mfma_f32_16x16x32_bf16 (or
// of four v_mfma_f32_16x16x4_f32) -- and goes from HBM to the matrix core through registers only.  The B
// operand is the activation block: staged in LDS, for bf16 weights as NSPLIT bfloat16 pieces x = x0 + x1 + x2
// (each product with a bf16 weight is then exact and the float32 accumulation sees the full float32
// activation), for f32 weights as float32.  When M rows of the reduction length do not fit in LDS the block is
// staged in activation tiles of KT8 blocks and the partial sums are carried in LDS between them.
//
// Every wave keeps RD (16, for prompt chunks 8) loads in flight in a register ring; a TURN of the ring is RD / 4
// blocks x 4 steps of one tile, set up once (all per-item cost is a clamp and an add).  The loader runs one turn
// ahead of the consumer over tile, group and PHASE boundaries (the weight addresses of later phases depend on no
// activation), so a phase starts with its first turn already in registers.  Load issue is throttled by the
// memory system (under load a turn takes one memory latency, 4-5 us, whether or not its data was prefetched), so
// the ring hides the ramp-up and the tail of a phase; across the boundary between two phases HBM stays busy only
// for as long as the one turn per wave that is in flight lasts.
//
// Row invariance: output column m of an MFMA depends on column m of B only; the order of steps per wave,
// the order of the pieces and the order in which the 8 wave partials are added are fixed.  Nothing depends
// on how many rows share the launch, so a verify row equals the one-row decode of the same prefix bit for bit.
#pragma once
#include "sdfp_common.hip.h"

namespace sdfp {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int RING_MAX = 16;                // deepest ring: 16-byte loads in flight per lane (1 KB per wave each)
constexpr int NSPLIT = 3;                  // bfloat16 pieces per float32 activation (bf16 weights)
constexpr int TG_MAX = 8;                  // tiles of a workgroup reduced together (a "group")
constexpr int STEP_BYTES = 64;             // bytes of one weight row consumed per step
constexpr int SPW = 4;                     // consecutive steps a wave takes from every weight row (256 B per row)
static_assert(SPW == 4, "item -> step mapping uses shifts by 2");
constexpr int BLOCK_STEPS = NWAVE * SPW;   // steps of a block: every wave's SPW steps, side by side
constexpr int BLOCK_BYTES = BLOCK_STEPS * STEP_BYTES;   // 2 KB of a weight row
constexpr int LDS_DYN_BYTES = 160 * 1024 - 1024;   // dynamic LDS of the forward kernel
constexpr int LDS_GEOM_OFF = LDS_DYN_BYTES - 512;  // Geom[8]: this workgroup's geometry per phase kind, kept for the launch
constexpr int LDS_ZERO_BYTES = NWAVE * SPW * STEP_BYTES;   // 2 KB of zeros: the activation operand of a ring slot that holds
constexpr int LDS_ZERO_OFF = LDS_GEOM_OFF - LDS_ZERO_BYTES;   // no block of the tile (every wave reads its own 256 bytes)
constexpr int XROW_PAD = 16;               // bytes added to every staged activation row (bank spread)
constexpr int SERVICE_WAVE = NWAVE - 1;    // the wave that runs epilogues, waits for their stores and passes barriers
constexpr int STAGE_THREADS = WG_THREADS - 64;   // the other waves stage activations (the service wave is the last; its
                                                 // loads would return behind the weights it has just asked for)

// ---- LDS map of a projection phase (bytes) ---------------------------------------------------------------
constexpr int LM_RS = 0;                       // float[16]     reciprocal RMS per row
constexpr int LM_SS = 64;                      // float[8][16]  per-wave sums of squares
constexpr int LM_BESTV = 576;                  // float[16]     running arg-max value per row (output head)
constexpr int LM_BESTI = 640;                  // int[16]
constexpr int LM_LG = 1024;                    // float[16][TG_MAX*16] logits of the current group (output head), or
                                               // the staged epilogue inputs of the group (residual / rotary rows)
constexpr int LM_MISC_BYTES = LM_LG + 16 * TG_MAX * 16 * 4;   // 9216
// then: red  float4[8 waves][TG][M][4]   wave partials of the group;   then: the staged activation block

enum { PK_END = 0, PK_EMBED, PK_QKV, PK_ATTN, PK_OPROJ, PK_GATEUP, PK_DOWN, PK_HEAD, PK_HOLD };

// One phase of a forward.  The host writes the phase list of the target model and of the draft model (the
// same list without the skipped sub-layers) once.  Between two phases the rows travel across a grid barrier or are
// handed over by the data itself (see Forward::POLL).
struct Phase {
    int kind, layer;
    int Kd;             // reduction length (projection kinds)
    int N;              // output features of the projection (QKV: (H + 2 Hkv) * hd; gate/up: F)
    int n_units;        // distribution units: QKV blocks of 8 rotary pairs, gate/up pairs, else output rows
    int pad_;
    const void* wt;     // the projection's matrices once more in tile order (tile t, step s -> one kilobyte, lane l's
                        // 16 bytes of the A operand at l * 16), or nullptr.  Only set where every workgroup's tiles are
                        // whole tiles of that numbering (O / down when N / 16 divides by the grid size; QKV could be).
    const void* w[3];   // QKV: wq wk wv; gate/up: w_gate w_up; else the matrix in w[0]
    const float* gain;  // RMSNorm gain applied to the input, or nullptr
    const float* xin;   // input rows [M][Kd] (ATTN: q)
    const float* res;   // residual input [M][N] (O / down projection)
    float* out;         // QKV: q [M][H*hd]; O / down: new residual [M][N]; gate/up: [M][F]; ATTN: [M][H*hd];
                        // EMBED: [M][d]
    void *kc, *vc;      // QKV / ATTN: this layer's key and value planes [Hkv][max_seq][hd]
};

// wave-uniform copy of a descriptor through the scalar data path
__device__ __forceinline__ Phase load_phase(const Phase* prog, int ph) {
    const SDFP_CONST Phase* q = as_const(prog) + ph;   // member by member: each access keeps its own type
    Phase p;
    p.kind = q->kind; p.layer = q->layer; p.Kd = q->Kd; p.N = q->N; p.n_units = q->n_units;
    p.pad_ = 0; p.wt = q->wt;
    p.w[0] = q->w[0]; p.w[1] = q->w[1]; p.w[2] = q->w[2];
    p.gain = q->gain; p.xin = q->xin; p.res = q->res; p.out = q->out;
    p.kc = q->kc; p.vc = q->vc;
    return p;
}

__device__ __forceinline__ bool is_projection(int kind) {
    return kind == PK_QKV || kind == PK_OPROJ || kind == PK_GATEUP || kind == PK_DOWN || kind == PK_HEAD;
}

// where the output projection puts its results
struct HeadOut {
    float* logits;        // [M][V] or nullptr
    float* part_val;      // [n_wg][MAX_ROWS]
    int* part_idx;        // [n_wg][MAX_ROWS]
    int dst;              // ROWS_DRAFT: st->d[off] ; otherwise st->amax[m]
    int off;
};

template <typename WT> struct XGeo;
template <> struct XGeo<bf16_t> { static constexpr int XROWS = NSPLIT; };   // LDS rows per activation row
template <> struct XGeo<float> { static constexpr int XROWS = 1; };

// ---- geometry of a projection phase for one workgroup ------------------------------------------------------
// Work is dealt out in UNITS so that every workgroup streams the same number of weight bytes (to within one
// unit): a unit is an output row (O / down projection, output head), a (gate row, up row) pair, or -- for
// QKV, whose tiles must not straddle heads -- a block of 8 rotary pairs.  A workgroup's units [u0, u1) are
// covered by tiles of `upt` units; the lanes of a last, partial tile re-read the workgroup's last unit (same
// cache lines, no extra HBM traffic) and their outputs are dropped.
struct Geom {
    int u0, u1;      // this workgroup's units
    int nt;          // its tiles
    int S;           // steps per weight row
    int nblk;        // blocks of BLOCK_STEPS steps covering the row
    int KT8;         // blocks per staged activation tile
    int TG;          // tiles per group
    int M;           // activation rows
    int red_off, xs_off, stride;   // LDS byte offsets / bytes per staged row
    int n_kt;        // staged activation tiles covering the row
    int pad_[3];     // 60 bytes
};

__device__ __forceinline__ int units_per_tile(int kind) { return kind == PK_QKV ? 1 : (kind == PK_GATEUP ? 8 : 16); }

template <typename WT>
__device__ __forceinline__ Geom make_geom(int kind, int n_units, int Kd, int M, int wg, int n_wg) {
    Geom g;
    g.u0 = (int)(((unsigned)n_units * (unsigned)wg) / (unsigned)n_wg);   // n_units * n_wg < 2^31
    g.u1 = (int)(((unsigned)n_units * (unsigned)(wg + 1)) / (unsigned)n_wg);
    const int upt = units_per_tile(kind);
    g.nt = (g.u1 - g.u0 + upt - 1) / upt;
    g.S = (Kd * (int)sizeof(WT)) / STEP_BYTES;
    g.nblk = (g.S + BLOCK_STEPS - 1) / BLOCK_STEPS;
    g.M = M;
    const int tgm = M > 8 ? TG_MAX / 2 : TG_MAX;
    g.TG = g.nt < tgm ? (g.nt > 0 ? g.nt : 1) : tgm;
    g.red_off = LM_MISC_BYTES;
    const int rows = M * XGeo<WT>::XROWS;
    auto blocks_that_fit = [&](int tg) { return ((LDS_ZERO_OFF - (g.red_off + NWAVE * tg * M * 64)) / rows - XROW_PAD) / BLOCK_BYTES; };
    // The wave partials of a group of TG tiles and the activation block share LDS.  Smaller groups (more epilogues
    // per phase) are much cheaper than staging the activations in tiles, so where the whole block fits next to a
    // smaller group, the group shrinks (six rows of 4096 bf16 columns fit next to one tile's partials, not eight).
    if (blocks_that_fit(g.TG) < g.nblk)
        for (int tg = g.TG / 2; tg >= 1; tg /= 2)
            if (blocks_that_fit(tg) >= g.nblk) { g.TG = tg; break; }
    g.xs_off = g.red_off + NWAVE * g.TG * M * 64;
    int kt8 = blocks_that_fit(g.TG);
    g.KT8 = kt8 < g.nblk ? kt8 : g.nblk;
    g.stride = g.KT8 * BLOCK_BYTES + XROW_PAD;
    g.n_kt = g.KT8 > 0 ? (g.nblk + g.KT8 - 1) / g.KT8 : 0;
    return g;
}

// The table entry of a kind, written once at the start of the launch, as wave-uniform values: a phase then costs a
// few LDS reads instead of make_geom's divisions, which sat between every two phases.
__device__ __forceinline__ Geom load_geom(const char* lds, int kind) {
    const Geom* t = reinterpret_cast<const Geom*>(lds + LDS_GEOM_OFF) + kind;
    Geom g;
    g.u0 = __builtin_amdgcn_readfirstlane(t->u0); g.u1 = __builtin_amdgcn_readfirstlane(t->u1);
    g.nt = __builtin_amdgcn_readfirstlane(t->nt); g.S = __builtin_amdgcn_readfirstlane(t->S);
    g.nblk = __builtin_amdgcn_readfirstlane(t->nblk); g.KT8 = __builtin_amdgcn_readfirstlane(t->KT8);
    g.TG = __builtin_amdgcn_readfirstlane(t->TG); g.M = __builtin_amdgcn_readfirstlane(t->M);
    g.red_off = __builtin_amdgcn_readfirstlane(t->red_off); g.xs_off = __builtin_amdgcn_readfirstlane(t->xs_off);
    g.stride = __builtin_amdgcn_readfirstlane(t->stride); g.n_kt = __builtin_amdgcn_readfirstlane(t->n_kt);
    return g;
}

// rows of this phase's forward: the output head may look at the last rows only
__device__ __forceinline__ int phase_rows(int kind, int M, int head_row_from) {
    return kind == PK_HEAD ? M - head_row_from : M;
}

// RD = ring depth (loads in flight per lane); a turn of the ring is RD / SPW blocks x SPW steps of one tile
template <int RD> struct Ring { u32x4 r[RD]; };


// One turn of the ring: RD loads, TURN_BLOCKS blocks x SPW steps.  The blocks come from one tile, or -- when that
// tile ends inside the turn and another tile of the same group and activation tile follows -- the first nA from
// the end of one tile and the rest from the start of the next (a row of five blocks would otherwise leave three
// quarters of every second turn empty).  Item j reads SPW consecutive steps (whole 128-byte lines) of block
// j / SPW: byte offset off0 + (j / SPW) * BLOCK_BYTES + (j % SPW) * STEP_BYTES from the lane's row pointer,
// clamped to `lim` -- the wave's last valid step of the segment -- so that a padding item re-reads a line that an
// earlier item of the turn fetched.  Everything but the row pointers is wave-uniform.
struct Turn {
    const char* rowp;       // per lane: its row of the (first) tile + 16 * (lane / 16)
    const char* rowp2;      // the same for the second tile (== rowp when the turn has one segment)
    int nA;                 // blocks of the first segment
    int span;               // 1 if there is a second segment
    int off0, lim;          // first segment
    int off2, lim2;         // second segment (a copy of the first when there is none: padding re-reads it)
    int sh;                 // log2 of the bytes of the matrix per byte of offset: 0 row-major (an offset is a byte of the
                            // lane's row), 4 tile order (a 64-byte step of a tile is a kilobyte)
    const char *lo, *hi;    // guard build: the matrix the first segment's row belongs to
    const char *lo2, *hi2;  // ... the second's
};

// ---- loader: walks the turn sequence of this wave over the whole phase list --------------------------------
// Order inside a phase: for group { for activation tile { for tile of the group { for turn } } }.  The consumer
// walks the same sequence one turn behind.  All bookkeeping happens once per turn; an item costs one scalar
// min, one address add and the load.
// SPAN: turns may go on into the next tile (see Turn); costs a few scalar operations per item, so only shapes whose
// rows do not fill whole turns use it
template <typename WT, int RD, bool SPAN>
struct Loader {
    static constexpr int TURN_BLOCKS = RD / SPW;
    const Phase* prog;
    const char* lds;
    int hd, H, Hkv;
    int head_run, wave;
    int ph, kind;                 // phase the loader is in; PK_END once the list is exhausted
    int pitch;                    // bytes per weight row
    int hold;                     // service wave: 1 = stop at every phase end until release(), 2 = only after a QKV phase
                                  // (where a grid barrier follows and its stores have to be waited for)
    const char *w0, *whi;         // matrices of the first / second half of a tile's rows (gate/up: w_gate, w_up)
    const char* wt;               // the phase's matrices in tile order, or nullptr (see Phase)
    int tmul, hioff, qsh;         // rows per tile step, row offset of the second half, log2(tiles per head)
    int u0, u1, nt, S, nblk, KT8, TG;   // this workgroup's geometry of the phase
    int grp0, grp_n, kt0, kt_n, t, c;   // group (first tile, tiles), activation tile (first block, blocks), tile, block
    const char* rowp;             // per lane: address of this lane's 16 bytes of step 0 of its row of tile t
    const char *mat_lo, *mat_hi;  // the matrix that row belongs to (guard build: exact bounds of the loads)
    int n_rows;                   // rows of a non-QKV matrix (guard build)
    int n_probe;                  // probe build: loads recorded so far

    // Address of this lane's row of tile t.  Written without per-kind branches and without selects between
    // struct members: branches once compiled into a path with an undefined base pointer, and a select among
    // adjacent members becomes a dynamically indexed access that keeps the whole loader in scratch memory.
    __device__ __forceinline__ void set_tile() {
        const int lane = threadIdx.x & 63, r = lane & 15, gq = lane >> 4;
        const bool hi = (r >> 3) != 0;            // second half of the tile's rows
        const int tl = grp0 + t;
        const bool isq = kind == PK_QKV;
        // QKV: unit = tile -> (head slot, 8 rotary pairs); rows (i, i + hd/2) of one head of wq, wk or wv.  The
        // matrix is fetched from the descriptor with a wave-uniform index (a scalar load from constant memory).
        const int tile = u0 + tl;
        const int hs = tile >> qsh, jj = tile - (hs << qsh);
        const int sel = isq ? (hs < H ? 0 : (hs < H + Hkv ? 1 : 2)) : 0;
        const int head = hs - (sel == 0 ? 0 : (sel == 1 ? H : H + Hkv));
        const char* qbase = (const char*)(as_const(prog) + ph)->w[sel];
        const int qrow = head * hd + jj * 8 + (r & 7) + (hi ? (hd >> 1) : 0);
        // other kinds: unit u0 + tl * tmul + (r & 7) + (hi ? hioff : 0), clamped to the workgroup's last unit,
        // of w0 (first half of the tile) or whi (second half)
        const int lrow = min(u0 + tl * tmul + (r & 7) + (hi ? hioff : 0), u1 - 1);
        const int row = isq ? qrow : lrow;
        const char* hbase = hi ? whi : w0;
        const char* base = isq ? qbase : hbase;
        // tile order: the workgroup's tile tl is tile (QKV: u0 + tl, else u0 / 16 + tl) of the copy; a step of it is a
        // kilobyte, this lane's 16 bytes at lane * 16.  Contiguous kilobytes cost the first-level cache 8 accesses
        // where a step read row by row costs 64; the down projection's stream (long rows) runs 15 % faster for it.
        const int gtile = isq ? tile : (u0 >> 4) + tl;
        const char* trow = wt + (size_t)gtile * (size_t)(S * 1024) + lane * 16;
        rowp = wt != nullptr ? trow : base + (size_t)row * (size_t)pitch + gq * 16;
#ifdef SDFP_GUARD
        const int nrows = isq ? (sel == 0 ? H : Hkv) * hd : n_rows;
        mat_lo = wt != nullptr ? wt : base;
        mat_hi = wt != nullptr ? wt + (size_t)(isq ? (H + 2 * Hkv) * (hd >> 4) : n_rows >> 4) * (size_t)(S * 1024)
                               : base + (size_t)nrows * (size_t)pitch;
#endif
    }
    __device__ __forceinline__ void set_group() {
        grp_n = min(TG, nt - grp0);
        kt0 = 0; kt_n = min(KT8, nblk);
        t = 0; c = 0;
    }
    // move to the next projection phase that has tiles for this workgroup
    __device__ __forceinline__ void next_phase() {
        for (;;) {
            ++ph;
#ifdef SDFP_GUARD
            if ((const void*)prog != s_guard.prog || ph < 0 || ph >= s_guard.prog_len) {   // never walk off the list
                guard_fail(prog + ph, ph, 50);
                kind = PK_END;
                return;
            }
#endif
            const SDFP_CONST Phase* p = as_const(prog) + ph;
            kind = p->kind;
            if (kind == PK_HEAD && !head_run) kind = PK_END;
            if (kind == PK_END) return;
            if (!is_projection(kind)) continue;
            const Geom* g = reinterpret_cast<const Geom*>(lds + LDS_GEOM_OFF) + kind;
            nt = __builtin_amdgcn_readfirstlane(g->nt);
            if (nt <= 0) continue;
            u0 = __builtin_amdgcn_readfirstlane(g->u0);
            u1 = __builtin_amdgcn_readfirstlane(g->u1);
            S = __builtin_amdgcn_readfirstlane(g->S);
            nblk = __builtin_amdgcn_readfirstlane(g->nblk);
            KT8 = __builtin_amdgcn_readfirstlane(g->KT8);
            TG = __builtin_amdgcn_readfirstlane(g->TG);
            pitch = p->Kd * (int)sizeof(WT); n_rows = p->N;
            wt = (const char*)p->wt;
            const bool gu = kind == PK_GATEUP;
            w0 = (const char*)p->w[0];
            whi = (const char*)p->w[gu ? 1 : 0]; tmul = gu ? 8 : 16; hioff = gu ? 0 : 8;
            grp0 = 0;
            set_group();
            set_tile();
            return;
        }
    }
    __device__ __forceinline__ void init(const Phase* prog_, const char* lds_, const LayerDims& L, int head_run_,
                                         int wave_, int hold_) {
        prog = prog_; lds = lds_; hd = L.hd; H = L.H; Hkv = L.Hkv; head_run = head_run_; wave = wave_; hold = hold_;
        qsh = 31 - __builtin_clz(hd) - 4;
        w0 = whi = nullptr; wt = nullptr; tmul = 16; hioff = 8; pitch = 0; n_rows = 1; u0 = 0; u1 = 1;
        ph = -1; kind = PK_HOLD;
        rowp = (const char*)prog_; mat_lo = nullptr; mat_hi = nullptr; n_probe = 0;
        S = 1; kt0 = 0; c = 0; kt_n = 1; grp_n = 1; t = 0; nblk = 1; KT8 = 1; TG = 1; nt = 0; grp0 = 0;
        if (!hold) next_phase();
    }
    // service wave: step from a phase end (or the start of the list) into the next phase with work
    __device__ __forceinline__ void release() {
        if (kind == PK_HOLD) next_phase();
    }
    // The current turn; the loader steps to the next one.  When there is nothing to fetch (hold, end of the list)
    // the turn re-reads the first 16 bytes of the phase list, a cached line: loads stay UNCONDITIONAL, so that the
    // turn body is straight-line code with one counted wait (a conditional load makes the compiler wait for
    // everything outstanding at each join).
    // Step to the next tile of the sequence.  True if it lies in the same group and activation tile, so that a
    // turn may go on into it.
    __device__ __forceinline__ bool next_tile() {
        c = 0;
        if (++t == grp_n) {   // next activation tile / group / phase
            t = 0;
            kt0 += kt_n;
            if (kt0 >= nblk) {
                grp0 += grp_n;
                if (grp0 >= nt) {
                    if (hold == 1 || (hold == 2 && kind == PK_QKV)) kind = PK_HOLD; else next_phase();
                    return false;
                }
                set_group();
            } else {
                kt_n = min(KT8, nblk - kt0);
            }
            set_tile();
            return false;
        }
        set_tile();
        return true;
    }
    __device__ __forceinline__ Turn next_turn() {
        Turn tr;
        if (kind == PK_END || kind == PK_HOLD) {
            tr.rowp = tr.rowp2 = (const char*)prog; tr.nA = TURN_BLOCKS; tr.span = 0; tr.off0 = tr.off2 = 0; tr.lim = tr.lim2 = 0;
            tr.sh = 0;
            tr.lo = tr.lo2 = (const char*)prog; tr.hi = tr.hi2 = (const char*)prog + 16;
            return tr;
        }
        const int nbA = min(TURN_BLOCKS, kt_n - c);
        tr.rowp = rowp; tr.lo = mat_lo; tr.hi = mat_hi;
        tr.nA = nbA; tr.span = 0; tr.sh = wt != nullptr ? 4 : 0;
        tr.off0 = (kt0 + c) * BLOCK_BYTES + wave * (SPW * STEP_BYTES);
        tr.lim = min((S - 1) * STEP_BYTES, tr.off0 + (nbA - 1) * BLOCK_BYTES + (SPW - 1) * STEP_BYTES);
        tr.rowp2 = tr.rowp; tr.off2 = tr.off0; tr.lim2 = tr.lim; tr.lo2 = tr.lo; tr.hi2 = tr.hi;
        c += nbA;
        if (c >= kt_n && next_tile() && SPAN && nbA < TURN_BLOCKS) {   // the turn goes on into the next tile
            const int nbB = min(TURN_BLOCKS - nbA, kt_n);
            tr.span = 1;
            tr.rowp2 = rowp; tr.lo2 = mat_lo; tr.hi2 = mat_hi;
            tr.off2 = kt0 * BLOCK_BYTES + wave * (SPW * STEP_BYTES);
            tr.lim2 = min((S - 1) * STEP_BYTES, tr.off2 + (nbB - 1) * BLOCK_BYTES + (SPW - 1) * STEP_BYTES);
            c = nbB;
            if (c >= kt_n) next_tile();
        }
        return tr;
    }
    // issue item j of a turn that has one segment (the common case, kept as cheap as it can be: the per-item
    // work competes with the matrix-core steps for issue slots)
    __device__ __forceinline__ u32x4 load_single(const Turn& tr, int j) {
        const int off = min(tr.off0 + (j / SPW) * BLOCK_BYTES + (j % SPW) * STEP_BYTES, tr.lim);
        const char* addr = tr.rowp + ((size_t)off << tr.sh);
#ifdef SDFP_PROBE
        if (tr.lim != 0 && s_guard.probe != nullptr && (threadIdx.x & 63) == 0 && n_probe < PROBE_N)
            __hip_atomic_store(s_guard.probe + (size_t)(blockIdx.x * 8 + wave) * PROBE_N + n_probe,
                               (unsigned long long)addr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if (tr.lim != 0) ++n_probe;
#endif
        return ld_stream(addr, tr.lo, tr.hi);
    }
    // issue item j of a turn
    __device__ __forceinline__ u32x4 load(const Turn& tr, int j) {
        if constexpr (!SPAN) return load_single(tr, j);
        const int b = j / SPW;
        const bool second = b >= tr.nA;   // wave-uniform
        const int off = second ? min(tr.off2 + (b - tr.nA) * BLOCK_BYTES + (j % SPW) * STEP_BYTES, tr.lim2)
                               : min(tr.off0 + b * BLOCK_BYTES + (j % SPW) * STEP_BYTES, tr.lim);
        const char* addr = (second ? tr.rowp2 : tr.rowp) + ((size_t)off << tr.sh);
#ifdef SDFP_PROBE
        if (tr.lim != 0 && s_guard.probe != nullptr && (threadIdx.x & 63) == 0 && n_probe < PROBE_N)
            __hip_atomic_store(s_guard.probe + (size_t)(blockIdx.x * 8 + wave) * PROBE_N + n_probe,
                               (unsigned long long)addr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if (tr.lim != 0) ++n_probe;
#endif
        return ld_stream(addr, second ? tr.lo2 : tr.lo, second ? tr.hi2 : tr.hi);
    }
};

// ---- matrix-core step: acc[16 rows][16 columns] += W step (A) x activation step (B) ------------------------
template <typename WT> struct Mma;
template <> struct Mma<bf16_t> {
    static __device__ __forceinline__ void run(f32x4& acc, const u32x4& a, const char* xl, int piece_stride) {
        const bf16x8 av = __builtin_bit_cast(bf16x8, a);
#pragma unroll
        for (int s = 0; s < NSPLIT; ++s) {
            const u32x4 b = *reinterpret_cast<const u32x4*>(__builtin_assume_aligned(xl + s * piece_stride, 16));
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
        }
    }
};
template <> struct Mma<float> {
    static __device__ __forceinline__ void run(f32x4& acc, const u32x4& a, const char* xl, int) {
        const f32x4 b = *reinterpret_cast<const f32x4*>(__builtin_assume_aligned(xl, 16));
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), b.x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), b.y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), b.z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), b.w, acc, 0, 0, 0);
    }
};

// write 8 consecutive activation values of one row into the staged block
template <typename WT> struct XStore;
template <> struct XStore<bf16_t> {
    static __device__ __forceinline__ void put(char* row0, int piece_stride, int k_rel, const float (&x)[8]) {
        split3_bf16_each(x, [&](int s, const u32x4& pk) {
            *reinterpret_cast<u32x4*>(__builtin_assume_aligned(row0 + s * piece_stride + k_rel * 2, 16)) = pk;
        });
    }
};
template <> struct XStore<float> {
    static __device__ __forceinline__ void put(char* row0, int, int k_rel, const float (&x)[8]) {
        f32x4* o = reinterpret_cast<f32x4*>(__builtin_assume_aligned(row0 + k_rel * 4, 16));
        o[0] = f32x4{x[0], x[1], x[2], x[3]};
        o[1] = f32x4{x[4], x[5], x[6], x[7]};
    }
};

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

// ---- one projection phase of one workgroup -----------------------------------------------------------------
// ROWS = the number of activation rows when the instance knows it at compile time (draft, plain decode: 1; a verify
// kernel per K + 1), or 0 = any, found in the geometry (prompt chunks).  A known row count compiles only the staging
// variant it needs and folds the divisions and loops over rows.
// POLL: the input rows are handed over by the data itself (no grid barrier precedes the phase).  Row 0 is armed
// at the start of the launch; a reader polls it with device-coherent loads until none of its values is still
// armed.  A writer stores its values of rows 1.. first, waits for their acknowledgement, and stores row 0 last:
// whoever has seen a stretch of row 0 written knows that the writers of those columns are done with every row, and
// only then reads the same columns of rows 1.. with plain loads, which the XCD's cache may serve to all its
// workgroups (polling all rows coherently costs M x 16 KB of fabric traffic per workgroup and phase, which made
// five-row forwards slower than the grid barrier did).  The rule behind it: a cache line of rows 1.. may enter
// the cache only once every writer of that line is done, because nobody fetches it a second time.
template <typename WT, int ROWS, int RD, bool POLL, bool SPAN>
struct Projection {
    static constexpr int TURN_BLOCKS = RD / SPW;
    static constexpr int XROWS = XGeo<WT>::XROWS;
    const Phase& p;
    const LayerDims& L;
    char* lds;
    Geom g;
    int kind, wave, lane, pos0;
    float eps;
    const float *cosT, *sinT;
    const HeadOut& head;
    unsigned long long* trace;   // timeline of workgroup 0's service wave, or nullptr
    int* n_trace;
    int trace_cap;
    unsigned* bar;               // grid-barrier words: the sticky time-out flag lives there
    unsigned spin_limit;         // bound of a hand-over wait, in polls

    __device__ __forceinline__ Projection(const Phase& p_, const LayerDims& L_, char* lds_, const Geom& g_, int wave_,
                                          int pos0_, float eps_, const float* cosT_, const float* sinT_,
                                          const HeadOut& head_, unsigned long long* trace_, int* n_trace_, int trace_cap_,
                                          unsigned* bar_, unsigned spin_limit_)
        : p(p_), L(L_), lds(lds_), g(g_), kind(p_.kind), wave(wave_), lane(threadIdx.x & 63), pos0(pos0_),
          eps(eps_), cosT(cosT_), sinT(sinT_), head(head_), trace(trace_), n_trace(n_trace_), trace_cap(trace_cap_),
          bar(bar_), spin_limit(spin_limit_) {}

    // input rows: coherent loads for the polled row 0 (a cached copy of it may be stale), plain ones elsewhere
    template <bool COH>
    __device__ __forceinline__ f32x4 ld_x4(const float* q) const {
        if constexpr (COH) return ld_coh4(q);
        else return ld_act4(q);
    }
    // One more poll of a hand-over wait?  Wave-uniform.  The wait is bounded like the grid barrier's: past
    // spin_limit polls the sticky flag is raised, and a raised flag (by anyone) ends every later wait at once.
    __device__ __forceinline__ bool poll_again(unsigned& spins) const {
        ++spins;
        if (spins > spin_limit) {
            st_coh(bar + BAR_FLAG_OFF, 1u);   // every active lane stores the same word
            return false;
        }
        if ((spins & 63u) == 1u && ld_coh(reinterpret_cast<const int*>(bar + BAR_FLAG_OFF)) != 0) return false;
        __builtin_amdgcn_s_sleep(2);
        return true;
    }

    // sub-phase timeline entry: tag = 32 + kind * 4 + {0: first activation block staged, 1: all items done,
    // 2: epilogue stores issued}
    __device__ __forceinline__ void mark(int sub) const {
#ifdef SDFP_WAVETRACE
        if (trace != nullptr && lane == 0 && *n_trace < trace_cap / NWAVE)
            as_global(trace)[wave * (trace_cap / NWAVE) + (*n_trace)++] =
                ((unsigned long long)(sub >= 16 ? sub : 32 + kind * 4 + sub) << 56) | (wall_clock64() & 0x00FFFFFFFFFFFFFFull);
        return;
#endif
        if (trace != nullptr && blockIdx.x == 0 && threadIdx.x == SERVICE_WAVE * 64 && *n_trace < trace_cap &&
            SDFP_OK(trace + *n_trace, 8, 42))
            as_global(trace)[(*n_trace)++] = ((unsigned long long)(32 + kind * 4 + sub) << 56) |
                                             (wall_clock64() & 0x00FFFFFFFFFFFFFFull);
    }

    // activation rows of the phase: a compile-time 1 in the one-row kernels, so that the divisions and loops over
    // rows fold away
    __device__ __forceinline__ int rows() const {
        if constexpr (ROWS > 0) return ROWS;
        else return g.M;
    }

    __device__ __forceinline__ float* lds_f(int off) const { return reinterpret_cast<float*>(lds + off); }

    // Sum of squares of every input row in a fixed order: thread t < 448 adds the 8-value chunks c = t (mod 448) in
    // ascending order, lanes are folded by the DPP tree, waves are added in index order by finish_norm.
    template <bool PL>
    __device__ __forceinline__ void sumsq_rows(int m_lo, int m_hi) const {
        const int nchunk = p.Kd >> 3;
        for (int m = m_lo; m < m_hi; ++m) {
            float s = 0.f;
            for (int c = threadIdx.x; c < nchunk && wave != SERVICE_WAVE; c += STAGE_THREADS) {
                const float* src = p.xin + (size_t)m * p.Kd + c * 8;
                f32x4 a = ld_x4<PL>(src), b = ld_x4<PL>(src + 4);
                if constexpr (PL) {
                    unsigned spins = 0;
                    while (armed8(a, b) && poll_again(spins)) { a = ld_x4<PL>(src); b = ld_x4<PL>(src + 4); }
                }
                s = add_rn(s, sq8(a, b));
            }
            s = wave_sum_last(s);
            if (lane == 63) lds_f(LM_SS)[wave * 16 + m] = s;
        }
    }
    __device__ __forceinline__ void sumsq_pass() const {
        if constexpr (POLL) {
            sumsq_rows<true>(0, 1);
            if (rows() > 1) {
                __syncthreads();   // all of row 0 seen: every writer is done with every row
                sumsq_rows<false>(1, rows());
            }
        } else {
            sumsq_rows<false>(0, rows());
        }
    }
    __device__ __forceinline__ void finish_norm() const {   // after a barrier that follows the sums
        if (threadIdx.x < rows()) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < NWAVE; ++w) s = add_rn(s, lds_f(LM_SS)[w * 16 + threadIdx.x]);
            lds_f(LM_RS)[threadIdx.x] = rms_recip(s, p.Kd, eps);
        }
    }

    // Stage blocks [kt0, kt0 + kt_n) of the input (times the norm gain) into LDS; columns past Kd are zero.
    // RB rows x U chunks are in flight per thread, so that a one-row phase needs one memory round trip and a
    // verify phase two.  A row's squares are added chunk by chunk in ascending order whatever M is.
    // PL: 1 = the rows are polled (row 0 of a hand-over); 0 = read once with plain loads; 2 = read once, row 0 with
    // a coherent load (it is known to be complete, but a cached copy of it may be stale), the others plain.
    template <int RB, int U, int PL>
    __device__ __forceinline__ void stage_rows(int kt0, int kt_n, bool with_ss, int m_lo, int m_hi) const {
        constexpr int KPB = BLOCK_BYTES / (int)sizeof(WT);   // k values per block
        const int c_lo = (kt0 * KPB) >> 3, c_hi = ((kt0 + kt_n) * KPB) >> 3, c_valid = p.Kd >> 3;
        const int piece_stride = rows() * g.stride;
        for (int m0 = m_lo; m0 < m_hi; m0 += RB) {
            float s[RB];
#pragma unroll
            for (int r = 0; r < RB; ++r) s[r] = 0.f;
            for (int c0 = c_lo + threadIdx.x; c0 < c_hi && wave != SERVICE_WAVE; c0 += U * STAGE_THREADS) {
                f32x4 v0[RB][U], v1[RB][U], g0[U], g1[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = c0 + u * STAGE_THREADS;
                    const bool valid = c < c_hi && c < c_valid;
                    g0[u] = f32x4{1.f, 1.f, 1.f, 1.f}; g1[u] = g0[u];
#ifndef SDFP_PROBE
                    if (valid && p.gain != nullptr) { g0[u] = ld_g4(p.gain + c * 8); g1[u] = ld_g4(p.gain + c * 8 + 4); }
#endif
                }
                for (unsigned spins = 0;;) {   // hand-over by data: again until the wave's whole batch is written
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int c = c0 + u * STAGE_THREADS;
                        const bool valid = c < c_hi && c < c_valid;
#pragma unroll
                        for (int r = 0; r < RB; ++r) {
                            v0[r][u] = f32x4{0.f, 0.f, 0.f, 0.f}; v1[r][u] = f32x4{0.f, 0.f, 0.f, 0.f};
                            if (valid && m0 + r < m_hi) {
                                const float* src = p.xin + (size_t)(m0 + r) * p.Kd + c * 8;
                                if (PL == 1 || (PL == 2 && m0 + r == 0)) { v0[r][u] = ld_x4<true>(src); v1[r][u] = ld_x4<true>(src + 4); }
                                else { v0[r][u] = ld_x4<false>(src); v1[r][u] = ld_x4<false>(src + 4); }
                            }
                        }
                    }
                    if constexpr (PL != 1) break;
                    bool armed = false;
#pragma unroll
                    for (int u = 0; u < U; ++u)
#pragma unroll
                        for (int r = 0; r < RB; ++r) armed = armed || armed8(v0[r][u], v1[r][u]);
                    if (!__any(armed) || !poll_again(spins)) break;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = c0 + u * STAGE_THREADS;
                    if (c >= c_hi) continue;
#pragma unroll
                    for (int r = 0; r < RB; ++r) {
                        if (m0 + r >= m_hi) continue;
                        const f32x4 a = v0[r][u], b = v1[r][u];
                        s[r] = add_rn(s[r], sq8(a, b));
                        float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                        if (p.gain != nullptr) {
                            x[0] = mul_rn(x[0], g0[u].x); x[1] = mul_rn(x[1], g0[u].y);
                            x[2] = mul_rn(x[2], g0[u].z); x[3] = mul_rn(x[3], g0[u].w);
                            x[4] = mul_rn(x[4], g1[u].x); x[5] = mul_rn(x[5], g1[u].y);
                            x[6] = mul_rn(x[6], g1[u].z); x[7] = mul_rn(x[7], g1[u].w);
                        }
                        XStore<WT>::put(lds + g.xs_off + (m0 + r) * g.stride, piece_stride, (c - c_lo) * 8, x);
                    }
                }
            }
            if (with_ss) {
#pragma unroll
                for (int r = 0; r < RB; ++r) {
                    if (m0 + r >= m_hi) continue;
                    const float t = wave_sum_last(s[r]);
                    if (lane == 63) lds_f(LM_SS)[wave * 16 + m0 + r] = t;
                }
            }
        }
    }
    // first: these columns of the rows are staged for the first time in this phase, so the call has to wait for
    // them; the later calls for the same columns (further groups of tiles) find them complete
    __device__ __forceinline__ void stage(int kt0, int kt_n, bool with_ss, bool first) const {
        if constexpr (ROWS == 1) {
            stage_rows<1, 4, POLL ? 1 : 0>(kt0, kt_n, with_ss, 0, 1);
        } else if constexpr (ROWS >= 2 && POLL) {
            if (first) {
                stage_rows<1, 2, 1>(kt0, kt_n, with_ss, 0, 1);
                // No workgroup barrier as a rule: a wave polls and then reads the same 64-chunk (2 KB) stretches
                // of a row, whole 128-byte cache lines, and it leaves the poll only when all of them are written in
                // row 0 -- so the writers of every line it is about to read in rows 1.. are done, and no line of
                // those rows enters the cache before that.  Rows that are not a whole number of lines long share
                // lines with their neighbours: then every wave waits until the workgroup has seen all of row 0.
                if ((p.Kd & 31) != 0) __syncthreads();
                constexpr int REST = ROWS - 1;
                if constexpr (REST <= 2) stage_rows<REST, 2, 0>(kt0, kt_n, with_ss, 1, ROWS);
                else if constexpr (REST <= 5) stage_rows<REST, 1, 0>(kt0, kt_n, with_ss, 1, ROWS);
                else stage_rows<(REST + 1) / 2, 1, 0>(kt0, kt_n, with_ss, 1, ROWS);   // two batches
            } else {   // one round trip for all rows
                if constexpr (ROWS <= 6) stage_rows<ROWS, 1, 2>(kt0, kt_n, with_ss, 0, ROWS);
                else stage_rows<(ROWS + 1) / 2, 1, 2>(kt0, kt_n, with_ss, 0, ROWS);
            }
        } else {
            if (g.M == 1) stage_rows<1, 4, 0>(kt0, kt_n, with_ss, 0, 1);
            else if (g.M <= 4) stage_rows<4, 2, 0>(kt0, kt_n, with_ss, 0, g.M);
            else stage_rows<8, 1, 0>(kt0, kt_n, with_ss, 0, g.M);
        }
    }

    // ---- epilogue inputs of a group, staged in LDS by all threads at the start of the group so that the
    // epilogue itself issues no global load: residual values (O / down) or rotary rows (QKV) ------------------
    __device__ __forceinline__ void stage_ex(int grp0, int grp_n) const {
        float* ex = lds_f(LM_LG);
        if (kind == PK_OPROJ || kind == PK_DOWN) {
            const int r0 = g.u0 + grp0 * 16, cnt = min(grp_n * 16, g.u1 - r0);   // ex[m * 128 + j] = res[m][r0 + j]
            for (int e = threadIdx.x; e < rows() * (TG_MAX * 16) && wave != SERVICE_WAVE; e += STAGE_THREADS) {
                const int m = e >> 7, j = e & (TG_MAX * 16 - 1);
                // Hand-over by data: the writer of a column stores its row 0 last, so once row 0 of the column is
                // no longer armed (coherent load: a cached copy may be stale) every row of the column is final.
                // The residual rows are older than the phase's input rows, so this wait ends at once as a rule,
                // and it comes before the wait for the input rows, which hides it.
                if (j < cnt) {
                    const float* src = p.res + (size_t)m * p.N + r0 + j;
                    if constexpr (POLL) {
                        const float* src0 = p.res + r0 + j;
                        float v0 = ld_coh(src0);
                        unsigned spins = 0;
                        while (__any(__float_as_uint(v0) == HANDOVER_ARMED) && poll_again(spins)) v0 = ld_coh(src0);
                        // rows 1.. of these few columns by coherent loads as well: a plain load would bring in a
                        // whole line, half of which belongs to another writer that may not be done yet
                        ex[e] = m == 0 ? v0 : ld_coh(src);
                    } else {
                        ex[e] = ld_act(src);
                    }
                }
            }
        } else if (kind == PK_QKV) {
            const int half = L.hd >> 1, tph = L.hd >> 4;   // ex[((tl * 8 + pr) * M + m) * 2 + {cos, sin}]
            for (int e = threadIdx.x; e < grp_n * 8 * rows() && wave != SERVICE_WAVE; e += STAGE_THREADS) {
                const int m = e % rows(), q = e / rows(), pr = q & 7, tl = q >> 3;
                const int tile = g.u0 + grp0 + tl, hs = tile / tph, i = (tile - hs * tph) * 8 + pr;
                const size_t at = (size_t)(pos0 + m) * half + i;
                ex[e * 2] = ld_g(cosT + at);
                ex[e * 2 + 1] = ld_g(sinT + at);
            }
        }
    }

    // value of output row `row` of tile `tl` for activation row m = sum of the 8 wave partials, in wave order
    __device__ __forceinline__ float red_sum(int tl, int m, int row) const {
        const float* red = lds_f(g.red_off);
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < NWAVE; ++w) s = add_rn(s, red[((w * g.TG + tl) * rows() + m) * 16 + row]);
        return s;
    }

    // ---- epilogue of a group, run by the service wave alone (the only wave whose stores must be waited for) --
    __device__ __forceinline__ void epilogue(int grp0, int grp_n) const {
        const bool norm = p.gain != nullptr;
        const float* rs = lds_f(LM_RS);
        const float* ex = lds_f(LM_LG);
        if (kind == PK_HEAD) {
            float* lg = lds_f(LM_LG);
            for (int e = lane; e < grp_n * rows() * 16; e += 64) {
                const int row = e & 15, tl = (e >> 4) % grp_n, m = (e >> 4) / grp_n;
                float v = red_sum(tl, m, row);
                if (norm) v = mul_rn(v, rs[m]);
                lg[m * (TG_MAX * 16) + tl * 16 + row] = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the wave's own LDS writes, then its reads
            __builtin_amdgcn_wave_barrier();
            const int n0 = g.u0 + grp0 * 16, cnt = min(grp_n * 16, g.u1 - n0);
            for (int m = 0; m < rows(); ++m) {
                float bv = -INFINITY; int bi = 0x7FFFFFFF;
                for (int j = lane; j < cnt; j += 64) {
                    const float v = lg[m * (TG_MAX * 16) + j];
                    if (head.logits != nullptr && SDFP_OK(head.logits + (size_t)m * p.N + n0 + j, 4, 30))
                        as_global(head.logits)[(size_t)m * p.N + n0 + j] = v;
                    if (better(v, n0 + j, bv, bi)) { bv = v; bi = n0 + j; }
                }
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    const float v = __shfl_xor(bv, off); const int i = __shfl_xor(bi, off);
                    if (better(v, i, bv, bi)) { bv = v; bi = i; }
                }
                if (lane == 0) {
                    float* bvs = lds_f(LM_BESTV); int* bis = reinterpret_cast<int*>(lds + LM_BESTI);
                    if (better(bv, bi, bvs[m], bis[m])) { bvs[m] = bv; bis[m] = bi; }
                }
            }
            return;
        }
        // one output pair of the group: rows pr and pr + 8 of tile tl for activation row m; e = index into `ex`
        auto item = [&](int m, int q, int e) {
            const int pr = q & 7, tl = q >> 3;
            float a = red_sum(tl, m, pr), b = red_sum(tl, m, pr + 8);
            if (norm) { a = mul_rn(a, rs[m]); b = mul_rn(b, rs[m]); }
            if (kind == PK_QKV) {
                const int tile = g.u0 + grp0 + tl;
                const int half = L.hd >> 1, tph = L.hd >> 4, hs = tile / tph, i = (tile - hs * tph) * 8 + pr;
                const int pos = pos0 + m;
                if (hs < L.H + L.Hkv) {   // rotary: (a, b) -> (a cos - b sin, b cos + a sin)
                    rotary_pair(a, b, ex[e * 2], ex[e * 2 + 1]);
                }
                if (hs < L.H) {
                    float* o = p.out + (size_t)m * L.H * L.hd + (size_t)hs * L.hd;
                    st_coh(o + i, a); st_coh(o + i + half, b);
                } else {
                    const bool isk = hs < L.H + L.Hkv;
                    const int kvh = isk ? hs - L.H : hs - L.H - L.Hkv;
                    WT* o = reinterpret_cast<WT*>(isk ? p.kc : p.vc) + ((size_t)kvh * L.max_seq + pos) * L.hd;
                    ST<WT>::stc(o + i, a); ST<WT>::stc(o + i + half, b);
                }
            } else if (kind == PK_GATEUP) {
                const int j = g.u0 + (grp0 + tl) * 8 + pr;
                if (j < g.u1) st_coh(p.out + (size_t)m * p.N + j, swiglu(a, b));
            } else {   // O / down projection: residual add into the next residual buffer
                const int jl = tl * 16 + pr, n = g.u0 + grp0 * 16 + jl;
                if (n < g.u1) st_coh(p.out + (size_t)m * p.N + n, add_rn(ex[m * (TG_MAX * 16) + jl], a));
                if (n + 8 < g.u1) st_coh(p.out + (size_t)m * p.N + n + 8, add_rn(ex[m * (TG_MAX * 16) + jl + 8], b));
            }
        };
        if (POLL && rows() > 1 && kind != PK_QKV) {
            // rows handed over by data: rows 1.. first, their acknowledgement, row 0 last (see POLL above)
            const int rest = rows() - 1;
            for (int e = lane; e < grp_n * rest * 8; e += 64) item(1 + e % rest, e / rest, 0);
            stores_done();
            for (int e = lane; e < grp_n * 8; e += 64) item(0, e, 0);
        } else {
            for (int e = lane; e < grp_n * rows() * 8; e += 64) item(e % rows(), e / rows(), e);
        }
    }

    // The whole phase; the ring of every wave that is not on hold holds the wave's first turn on entry.  On return the service wave has
    // issued every store of the phase (it has not waited for them); the other waves have stored nothing.
    // ph: index of this phase in the list.
    __device__ __forceinline__ void run(Ring<RD>& ring, Loader<WT, RD, SPAN>& ld, int ph) const {
        if (g.nt <= 0) return;   // uniform over the workgroup
        const bool norm = p.gain != nullptr;
        const bool service = wave == SERVICE_WAVE;
        const int m_l = lane & 15, gq = lane >> 4;
        const int piece_stride = rows() * g.stride;
        const char* xl = lds + g.xs_off + (m_l < rows() ? m_l : 0) * g.stride + wave * (SPW * STEP_BYTES) + gq * 16;
        f32x4* red = reinterpret_cast<f32x4*>(lds + g.red_off);
        const char* xz = lds + LDS_ZERO_OFF + wave * (SPW * STEP_BYTES) + gq * 16;   // this lane's share of the zeros
        const int n_kt = g.n_kt;

        // The service wave's ring is empty wherever a grid barrier preceded the phase (it had to wait for its
        // stores, which on this hardware means for every load as well): it fetches the phase's first turn now.
        // The service wave's loader stops where a grid barrier follows (there the wave has to wait for its stores,
        // which on this hardware means for every load as well, so it must not have weights on their way).  The
        // loader runs one turn ahead of the consumer: it goes on hold when it hands out the last turn of such a
        // phase, so at the start of that very phase (ld.ph == ph) the ring may already hold the phase's first
        // turn, prefetched; at the start of a later phase the ring is empty and the first turn is fetched now.
        if (service && ld.kind == PK_HOLD && ld.ph != ph) {
            ld.release();
            const Turn t0 = ld.next_turn();
#pragma unroll
            for (int j = 0; j < RD; ++j) ring.r[j] = ld.load(t0, j);
        }
        if (kind == PK_HEAD && threadIdx.x < 16) {
            lds_f(LM_BESTV)[threadIdx.x] = -INFINITY;
            reinterpret_cast<int*>(lds + LM_BESTI)[threadIdx.x] = 0x7FFFFFFF;
        }
        if (norm && n_kt > 1) sumsq_pass();

        for (int grp0 = 0; grp0 < g.nt; grp0 += g.TG) {
            const int grp_n = min(g.TG, g.nt - grp0);
            if (grp0 > 0) __syncthreads();   // the previous group's epilogue has read its partials and inputs
#ifdef SDFP_WAVETRACE
            mark(19);
#endif
            stage_ex(grp0, grp_n);
#ifdef SDFP_WAVETRACE
            mark(20);
#endif
            for (int kt0 = 0; kt0 < g.nblk; kt0 += g.KT8) {
                const int kt_n = min(g.KT8, g.nblk - kt0);
                SDFP_BEACON2(10 + kt0 * 100 + grp0 * 100000);
                if (n_kt > 1 || grp0 == 0) {
                    if (kt0 > 0) __syncthreads();   // every wave is done with the previous block
                    // group 0 waits for the rows tile by tile: an activation tile's columns come from writers
                    // that no earlier tile's poll has covered; later groups find every tile complete
                    stage(kt0, kt_n, norm && n_kt == 1, grp0 == 0);
#ifdef SDFP_WAVETRACE
                    mark(21);
#endif
                    __syncthreads();
                    SDFP_BEACON2(11 + kt0 * 100 + grp0 * 100000);
                    if (norm && grp0 == 0 && kt0 == 0) finish_norm();   // read after the group's last barrier
                    if (grp0 == 0 && kt0 == 0) mark(0);
                }
                // The wave's turns of this (group, activation tile): for every tile, TURN_BLOCKS blocks at a time.
                // Slot j of the ring holds item j of the current turn and is refilled with item j of the loader's
                // next turn as soon as it is consumed.
                // The consumer mirrors the loader's rule for turns that go on into the next tile (see Turn).
                auto tile_init = [&](int tl) {
                    f32x4 a = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (kt0 > 0 && m_l < rows()) a = red[((wave * g.TG + tl) * rows() + m_l) * 4 + gq];
                    return a;
                };
                auto tile_store = [&](int tl, const f32x4& a) {   // this wave's share of the tile
                    if (m_l < rows()) red[((wave * g.TG + tl) * rows() + m_l) * 4 + gq] = a;
                };
                int tl = 0, c = 0;
                f32x4 acc = tile_init(0);
                while (tl < grp_n) {
                    const int nbA = min(TURN_BLOCKS, kt_n - c);
                    const bool more = SPAN && c + nbA >= kt_n && tl + 1 < grp_n && nbA < TURN_BLOCKS;
                    const int nbB = more ? min(TURN_BLOCKS - nbA, kt_n) : 0;
                    const Turn nx = ld.next_turn();
                    // consume slot j, THEN refill it: the new load may then target the same registers, so the
                    // ring needs no copy at the end of the turn.  The generated code waits once, at the top of the
                    // turn, for the 16 loads issued during the previous turn and then runs through the slots; with
                    // two waves per SIMD and 8 per workgroup that keeps enough loads in flight to stream at the
                    // memory's rate (a build with a third of the matrix-core work per slot streams no faster).
#pragma unroll
                    for (int j = 0; j < RD; ++j) {
                        const int b = j / SPW;
                        if (j % SPW == 0 && b > 0 && b == nbA && nbB > 0) {   // the next tile starts with this block
                            tile_store(tl, acc);
                            acc = tile_init(tl + 1);
                        }
                        // Every slot goes through the matrix core, without a branch (a branch would split the turn
                        // into pieces that each wait for all outstanding loads).  A slot that holds no block of the
                        // tile (its load re-read an earlier line) is multiplied by a block of zeros kept in LDS.
                        const int xb = b < nbA ? c + b : b - nbA;   // block of the activation tile
                        const bool real = b < nbA + nbB;
                        const char* xp = real ? xl + xb * BLOCK_BYTES : xz;
                        Mma<WT>::run(acc, ring.r[j], xp + (j % SPW) * STEP_BYTES, real ? piece_stride : 0);
                        ring.r[j] = ld.load(nx, j);
                    }
#ifdef SDFP_WAVETRACE
                    mark(17);
#endif
                    if (nbB > 0) { ++tl; c = nbB; } else { c += nbA; }
                    if (c >= kt_n) {
                        tile_store(tl, acc);
                        ++tl; c = 0;
                        if (tl < grp_n) acc = tile_init(tl);
                    }
                }
                SDFP_BEACON2(12 + kt0 * 100 + grp0 * 100000);
            }
#ifdef SDFP_WAVETRACE
            mark(16);
#endif
            __syncthreads();   // all partials of the group (and, for group 0, the reciprocal RMS) are in LDS
            SDFP_BEACON2(13 + grp0 * 100000);
            if (grp0 + g.TG >= g.nt) mark(1);
            if (service) epilogue(grp0, grp_n);
            if (grp0 + g.TG >= g.nt) mark(2);
            SDFP_BEACON2(14 + grp0 * 100000);
        }
        if (kind == PK_HEAD && service && lane < rows()) {   // this workgroup's arg-max partial per row
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            st_coh(head.part_val + (size_t)blockIdx.x * MAX_ROWS + lane, lds_f(LM_BESTV)[lane]);
            st_coh(head.part_idx + (size_t)blockIdx.x * MAX_ROWS + lane, reinterpret_cast<int*>(lds + LM_BESTI)[lane]);
        }
    }
};

// final reduce over the n_wg arg-max partials by one workgroup: wave m handles row m
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
            int* dst = out.dst == ROWS_DRAFT ? &st->d[out.off] : &st->amax[m];
            if (SDFP_OK(dst, 4, 31)) *as_global(dst) = bi;
        }
    }
}

}  // namespace sdfp
