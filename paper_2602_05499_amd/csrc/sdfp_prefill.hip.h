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
// Layout of a panel of P prompt rows in the workspace: h [P][d] float32 residual stream (updated in place); xs, the
// three bfloat16 pieces of the current projection input, each piece in OPERAND ORDER (pf_xs_off): the B operand of one
// matrix-core step -- 16 rows x 64 bytes -- is one contiguous kilobyte, lane l's 16 bytes at l * 16, so that the GEMM
// stages a slab with contiguous reads and writes it to LDS as it comes; q, att [P][H*hd] float32; rs [P] float32.
#pragma once
#include "sdfp_attn.hip.h"

namespace sdfp {

constexpr int PF_NSHARE = 8;             // shares of the reduction dimension (= waves of the decode kernels)
constexpr int PF_STEP_BYTES = 64;        // bytes of a weight row per matrix-core step (32 bfloat16)
constexpr int PF_SPS = 4;                // consecutive steps of a share per block
constexpr int PF_BLOCK_BYTES = PF_NSHARE * PF_SPS * PF_STEP_BYTES;   // 2 KB
constexpr int PF_TM = 64;                // prompt rows per workgroup tile
constexpr int PF_FRAG_BYTES = 16 * PF_STEP_BYTES;          // one B operand: a step of 16 prompt rows, lane l's 16 bytes at l * 16
constexpr int PF_SLAB_BYTES = 3 * (PF_TM / 16) * PF_SPS * PF_FRAG_BYTES;   // pieces x column tiles x steps: 48 KB
constexpr int PF_LDS_BYTES = 2 * PF_SLAB_BYTES;            // double-buffered

// Byte offset, inside one piece of an input with rows of Kd values, of the 16-byte unit that holds values 8 * k8 .. + 7 of
// row m: [16-row tile][64-byte step][quarter of the step][row of the tile][16 bytes].  A piece spans a whole number of
// tiles: ceil(rows / 16) * 16 * Kd values.
__host__ __device__ __forceinline__ size_t pf_xs_off(int m, int k8, int Kd) {
    return ((size_t)(m >> 4) * (size_t)(Kd >> 5) + (size_t)(k8 >> 2)) * PF_FRAG_BYTES + (size_t)((k8 & 3) * 256 + (m & 15) * 16);
}
__host__ __device__ __forceinline__ size_t pf_xs_piece(int rows, int Kd) { return (size_t)((rows + 15) / 16 * 16) * (size_t)Kd; }

enum { PF_QKV = 0, PF_OPROJ = 1, PF_GATEUP = 2, PF_DOWN = 3, PF_PLAIN = 4 };   // PF_PLAIN: out = (out +) x W^T, nothing fused

struct PfGemm {
    const bf16_t* w[3];      // QKV: wq wk wv; gate/up: w_gate w_up; else the matrix in w[0]; row-major [N][Kd]
    const bf16_t* wt;        // the projection's matrices once more in tile order (pf_tile_weights), or nullptr
    const bf16_t* xs;        // the three pieces of the input rows, each in operand order (pf_xs_off)
    size_t xs_piece;         // elements between pieces (pf_xs_piece)
    int Kd;                  // reduction length
    int n_tiles;             // 16-row weight tiles of the projection
    int M;                   // valid prompt rows of the panel
    int pos0;                // absolute position of the panel's row 0
    const float* rs;         // [P] reciprocal RMS of the input rows (QKV, gate/up), else nullptr
    float* h;                // O / down: residual stream [P][d], updated in place
    float* q;                // QKV: queries [P][H*hd]
    bf16_t *kc, *vc;         // QKV: this layer's key / value planes [Hkv][max_seq][hd]
    bf16_t* xs_out;          // gate/up: the pieces of the feed-forward activation (rows of F values), in operand order
    size_t xs_out_piece;
    const float *cosT, *sinT;
    float* out;              // PF_PLAIN: [M][ldo] float32 result
    int ldo;                 // PF_PLAIN: elements between rows of out
    int accumulate;          // PF_PLAIN: add to what out holds instead of overwriting it
    float* part;             // a projection dealt by shares: [8][P][part_ld] partial sums
    size_t part_arr;         // floats per array of part (P * part_ld)
    int part_ld;             // floats per row of part: the projection's outputs (16 * n_tiles)
    int n_nt;                // groups of 8 * NT weight tiles
    int my;                  // row tiles of the panel (64 rows each)
    int n_groups;            // workgroups that share a tile's reduction dimension: 1, 2, 4 or 8
    LayerDims L;
};

// ---- RMSNorm prologue of a projection, in two kernels.  k_pf_rownorm: the reciprocal RMS of every row from its sum of
// squares in the decode kernels' order -- one workgroup of 512 threads per prompt row; threads 0..447 are the decode
// kernels' staging threads: thread t adds the 8-value chunks t, t + 448, ... in ascending order, lanes are folded by
// the DPP tree, the eight wave sums are added in wave order (the last wave's is 0).  k_pf_split: the rows (times the
// gain, if any) split into pieces, written in operand order. ----------------------------------------------------------
__global__ __launch_bounds__(512) void k_pf_rownorm(const float* __restrict__ h, int d, float eps, float* __restrict__ rs) {
    __shared__ float ss[NWAVE];
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* row = h + (size_t)m * d;
    const int nchunk = d >> 3;
    float s = 0.f;
    for (int c = tid; c < nchunk && wave != NWAVE - 1; c += WG_THREADS - 64) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(row + c * 8), b = *reinterpret_cast<const f32x4*>(row + c * 8 + 4);
        s = add_rn(s, sq8(a, b));
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

// x [rows][Kd] float32 (times gain [Kd], or gain == nullptr) -> three pieces in operand order.  A wave takes a
// fragment -- a 64-byte step of a 16-row tile -- at a time: lane l reads the 8 values (l / 16) * 8 .. of the step of row
// l % 16 and writes its 16 bytes of each piece at l * 16 of the fragment, a contiguous kilobyte per piece.  Rows past
// the last one repeat it (a piece spans whole tiles; what those rows produce is never used).
__global__ __launch_bounds__(256) void k_pf_split(const float* __restrict__ x, const float* __restrict__ gain, int rows, int Kd,
                                                  bf16_t* __restrict__ xs, size_t xs_piece) {
    const int lane = threadIdx.x & 63, r16 = lane & 15, gq = lane >> 4;
    const int S = Kd >> 5, n_frag = ((rows + 15) >> 4) * S;
    for (int f = blockIdx.x * 4 + (threadIdx.x >> 6); f < n_frag; f += gridDim.x * 4) {
        const int t = f / S, st = f - t * S;
        const int m = min(t * 16 + r16, rows - 1), k0 = st * 32 + gq * 8;
        const float* src = x + (size_t)m * Kd + k0;
        const f32x4 a = *reinterpret_cast<const f32x4*>(src), b = *reinterpret_cast<const f32x4*>(src + 4);
        float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        if (gain != nullptr) {
            const f32x4 g0 = *reinterpret_cast<const f32x4*>(gain + k0), g1 = *reinterpret_cast<const f32x4*>(gain + k0 + 4);
            v[0] = mul_rn(v[0], g0.x); v[1] = mul_rn(v[1], g0.y); v[2] = mul_rn(v[2], g0.z); v[3] = mul_rn(v[3], g0.w);
            v[4] = mul_rn(v[4], g1.x); v[5] = mul_rn(v[5], g1.y); v[6] = mul_rn(v[6], g1.z); v[7] = mul_rn(v[7], g1.w);
        }
        u32x4 piece[3];
        split3_bf16(v, piece);
#pragma unroll
        for (int p = 0; p < 3; ++p)
            *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(xs + p * xs_piece) + (size_t)f * PF_FRAG_BYTES + lane * 16) = piece[p];
    }
}

// The three kernels that stand between two projections, in one: the residual update of a projection dealt by shares
// (h += ((((0 + P0) + P1) + ...) + P7), k_pf_residual; left out when part == nullptr), the reciprocal RMS of the new row
// (k_pf_rownorm: same threads, same chunks, same order) and the pieces of the row times the gain in operand order
// (k_pf_split).  One workgroup per prompt row; a thread keeps its chunks of the row in registers between the steps
// (rows of at most PF_FUSED_MAX_D values).  The rows that pad the last 16-row tile are left as they are, as the gate/up
// GEMM leaves them in the pieces it writes: an operand column feeds its own output column only, and those are dropped.
constexpr int PF_FUSED_CHUNKS = 3;                                   // 8-value chunks a thread may hold
constexpr int PF_FUSED_MAX_D = PF_FUSED_CHUNKS * 8 * (WG_THREADS - 64);
__global__ __launch_bounds__(512) void k_pf_residual_norm_split(float* __restrict__ h, const float* __restrict__ part, size_t part_arr,
                                                                int d, float eps, const float* __restrict__ gain,
                                                                float* __restrict__ rs, bf16_t* __restrict__ xs, size_t xs_piece) {
    __shared__ float ss[NWAVE];
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* row = h + (size_t)m * d;
    const int nchunk = d >> 3;
    float v[PF_FUSED_CHUNKS][8];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PF_FUSED_CHUNKS; ++i) {
        const int c = tid + i * (WG_THREADS - 64);
        if (c < nchunk && wave != NWAVE - 1) {
            f32x4 a = *reinterpret_cast<const f32x4*>(row + c * 8), b = *reinterpret_cast<const f32x4*>(row + c * 8 + 4);
            if (part != nullptr) {
                f32x4 ta = f32x4{0.f, 0.f, 0.f, 0.f}, tb = ta;
#pragma unroll
                for (int p = 0; p < PF_NSHARE; ++p) {
                    const float* src = part + (size_t)p * part_arr + (size_t)m * d + c * 8;
                    const f32x4 pa = *reinterpret_cast<const f32x4*>(src), pb = *reinterpret_cast<const f32x4*>(src + 4);
                    ta = f32x4{add_rn(ta.x, pa.x), add_rn(ta.y, pa.y), add_rn(ta.z, pa.z), add_rn(ta.w, pa.w)};
                    tb = f32x4{add_rn(tb.x, pb.x), add_rn(tb.y, pb.y), add_rn(tb.z, pb.z), add_rn(tb.w, pb.w)};
                }
                a = f32x4{add_rn(a.x, ta.x), add_rn(a.y, ta.y), add_rn(a.z, ta.z), add_rn(a.w, ta.w)};
                b = f32x4{add_rn(b.x, tb.x), add_rn(b.y, tb.y), add_rn(b.z, tb.z), add_rn(b.w, tb.w)};
                *reinterpret_cast<f32x4*>(row + c * 8) = a; *reinterpret_cast<f32x4*>(row + c * 8 + 4) = b;
            }
            s = add_rn(s, sq8(a, b));
            v[i][0] = a.x; v[i][1] = a.y; v[i][2] = a.z; v[i][3] = a.w; v[i][4] = b.x; v[i][5] = b.y; v[i][6] = b.z; v[i][7] = b.w;
        }
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
    const int S = d >> 5;                                            // 64-byte steps of a row of pieces
#pragma unroll
    for (int i = 0; i < PF_FUSED_CHUNKS; ++i) {
        const int c = tid + i * (WG_THREADS - 64);
        if (c < nchunk && wave != NWAVE - 1) {
            const f32x4 g0 = *reinterpret_cast<const f32x4*>(gain + c * 8), g1 = *reinterpret_cast<const f32x4*>(gain + c * 8 + 4);
            const float x[8] = {mul_rn(v[i][0], g0.x), mul_rn(v[i][1], g0.y), mul_rn(v[i][2], g0.z), mul_rn(v[i][3], g0.w),
                                mul_rn(v[i][4], g1.x), mul_rn(v[i][5], g1.y), mul_rn(v[i][6], g1.z), mul_rn(v[i][7], g1.w)};
            u32x4 piece[3];
            split3_bf16(x, piece);
            // chunk c = step c / 4, bytes (c % 4) * 16 .. of it: lane slot (c % 4) * 16 + row % 16 of the fragment
            const size_t at = ((size_t)(m >> 4) * S + (c >> 2)) * PF_FRAG_BYTES + (size_t)(((c & 3) << 4) + (m & 15)) * 16;
#pragma unroll
            for (int p = 0; p < 3; ++p) *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(xs + p * xs_piece) + at) = piece[p];
        }
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

// This lane's row (r16 = lane % 16) of weight tile t of a projection, in the caller's row-major matrices.
template <int KIND>
__device__ __forceinline__ const char* pf_weight_row(const PfGemm& a, int t, int r16) {
    const size_t pitch = (size_t)a.Kd * 2;
    const bool hi = r16 >= 8;
    if (KIND == PF_QKV) {          // tile = 8 rotary pairs of one head of wq, wk or wv: rows (i, i + hd / 2)
        const int hd = a.L.hd, H = a.L.H, Hkv = a.L.Hkv, tph = hd >> 4;
        const int hs = t / tph, jj = t - hs * tph;
        const int sel = hs < H ? 0 : (hs < H + Hkv ? 1 : 2);
        const int head = hs - (sel == 0 ? 0 : (sel == 1 ? H : H + Hkv));
        const int row = head * hd + jj * 8 + (r16 & 7) + (hi ? (hd >> 1) : 0);
        return (const char*)a.w[sel] + (size_t)row * pitch;
    }
    if (KIND == PF_GATEUP)         // tile = 8 gate rows and the 8 up rows of the same units
        return (const char*)a.w[hi ? 1 : 0] + (size_t)(t * 8 + (r16 & 7)) * pitch;
    return (const char*)a.w[0] + (size_t)(t * 16 + r16) * pitch;
}

// The matrices of a projection once more, in tile order: tile t, step s -> one kilobyte, lane l's 16 bytes of the A
// operand (row l % 16 of the tile, bytes (l / 16) * 16 .. of the step) at l * 16.  The GEMM then reads a step of a tile
// as one contiguous kilobyte.  Read row by row the same step is 64 separate 16-byte accesses of the first-level cache
// (adjacent lanes hold different rows), which that cache serves at about one per cycle: measured on resident data,
// 9.6 TB/s against 32 TB/s for contiguous kilobytes -- enough for a kernel bound by HBM, not for one whose weights come
// from the L2 cache eight times over.  a: w, Kd, n_tiles, L as for the GEMM.
template <int KIND>
__global__ __launch_bounds__(256) void k_pf_tile_weights(PfGemm a, bf16_t* __restrict__ dst) {
    const int lane = threadIdx.x & 63, r16 = lane & 15, gq = lane >> 4;
    const int S = a.Kd * 2 / PF_STEP_BYTES;
    const size_t n_frag = (size_t)a.n_tiles * S;
    for (size_t f = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6); f < n_frag; f += (size_t)gridDim.x * 4) {
        const int t = (int)(f / S), s = (int)(f - (size_t)t * S);
        const char* src = pf_weight_row<KIND>(a, t, r16) + s * PF_STEP_BYTES + gq * 16;
        *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(dst) + f * PF_FRAG_BYTES + lane * 16) =
            *reinterpret_cast<const u32x4*>(src);
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
// PARTIAL: the projection is too narrow to fill the chip with whole outputs (O and down projections; QKV of a short
// prompt), so the shares of the reduction dimension are dealt to n_groups workgroups per tile; each writes its shares'
// partial sums P_p to part[p][row][N], and k_pf_residual (k_pf_finish_qkv) adds them in share order.
// JT: 16-row column tiles of the workgroup tile that are multiplied (4; 1 or 2 for a panel of at most 16 or 32 rows,
// which then costs a quarter or half of the matrix-core instructions and LDS reads, and fetches as much less).
template <int KIND, int NT, bool PARTIAL, int JT = 4>
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

    // This lane's 16 bytes of step 0 of tile t (tiles past the end repeat the last one; their outputs are dropped), and
    // the bytes from one step to the next: in the tiled copy a step of a tile is a kilobyte, in the caller's matrices
    // 64 bytes of each of the tile's rows.
    const bool tiled = a.wt != nullptr;
    const int wstep = tiled ? PF_FRAG_BYTES : PF_STEP_BYTES;
    const char* wrow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tc = min(t0 + t, a.n_tiles - 1);
        wrow[t] = tiled ? (const char*)a.wt + (size_t)tc * S * PF_FRAG_BYTES + lane * 16
                        : pf_weight_row<KIND>(a, tc, r16) + gq * 16;
    }

    // Staging of a slab: 3 pieces x 64 prompt rows x 256 bytes = 48 fragments of 1 KB, 6 per wave.  The slab lies in LDS
    // as it lies in memory, in operand order: fragment f = (piece * 4 + column tile) * 4 + step, lane l's 16 bytes
    // (prompt row l % 16 of the column tile, bytes (l / 16) * 16 .. of the step) at l * 16 -- a wave reads a B operand
    // as one contiguous kilobyte, free of bank conflicts however the hardware groups the lanes, and a fragment travels
    // from memory to LDS with one load-to-LDS instruction per wave (lane l's 16 bytes land at l * 16), through no
    // register.
    const char* xs_base = (const char*)a.xs;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // slab i of the walk: share p = i / nblk, block b = i % nblk; its first byte in a row, and how many of its 4 steps exist
    auto slab_byte0 = [&](int i) { return (i % nblk) * PF_BLOCK_BYTES + (i / nblk) * (PF_SPS * PF_STEP_BYTES); };
    auto slab_steps = [&](int i) { return max(0, min(PF_SPS, S - ((i % nblk) * (PF_NSHARE * PF_SPS) + (i / nblk) * PF_SPS))); };
    const int spg = PF_NSHARE / a.n_groups;                 // shares per group
    const int i_lo = grp * spg * nblk, i_hi = i_lo + spg * nblk;

    f32x4 total[PARTIAL ? 1 : NT][PARTIAL ? 1 : JT], acc[NT][JT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int j = 0; j < JT; ++j) {
            acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (!PARTIAL) total[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    // Every load of the loop below is unconditional and its address clamped into the row: a load under a condition makes
    // the compiler wait, at the join, for everything in flight, and the pipeline (pieces and weights one slab ahead)
    // would stall once per step.  What a clamped load brings is never used: the steps a slab does not have are skipped.
    u32x4 wa[NT][PF_SPS];   // the wave's weight steps: of this slab until a step is multiplied, of the next one after
    const int last_tile16 = (a.M - 1) >> 4;
    // Slab i into LDS buffer buf; wave w fetches fragments w, w + 8, ...  The loads are counted with the wave's other
    // vector memory loads and complete in order with them.  They are issued from an asm statement: told what they are,
    // the compiler makes every later LDS read that it cannot prove disjoint (the other buffer) wait for them, i.e. for
    // all memory traffic of the wave, once per slab.  So the kernel waits for them itself, before the barrier that lets
    // anybody read the buffer; the compiler's own waits for the weight loads merely count up to 6 loads too few in
    // flight, which makes them wait for a little more than they need, never less.
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds;
    auto fetch_slab = [&](int i, int buf) {
        const int byte0 = slab_byte0(i);
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            const int frag = wave_u + u * NWAVE, piece = frag >> 4;
            if (JT < 4 && ((frag >> 2) & 3) >= JT) continue;   // a column tile that is not multiplied (wave-uniform)
            const int tile16 = min((m0 >> 4) + ((frag >> 2) & 3), last_tile16);
            const int step = min((byte0 >> 6) + (frag & 3), S - 1);
            const char* src = xs_base + (size_t)piece * a.xs_piece * 2 + ((size_t)tile16 * S + step) * PF_FRAG_BYTES + lane * 16;
            // M0 = LDS byte address of the fragment (wave-uniform); lane l's 16 bytes land at M0 + l * 16
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                         :
                         : "s"(lds0 + (unsigned)(buf * PF_SLAB_BYTES + frag * PF_FRAG_BYTES)), "v"(src)
                         : "memory");   // (M0 is not allocatable: the compiler sets it in front of each of its own uses)
        }
    };
    auto load_weight_step = [&](int byte0, int s) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
            wa[t][s] = *reinterpret_cast<const u32x4*>(wrow[t] + (size_t)(min((byte0 >> 6) + s, S - 1) * wstep));
    };

    fetch_slab(i_lo, 0);
#pragma unroll
    for (int s = 0; s < PF_SPS; ++s) load_weight_step(slab_byte0(i_lo), s);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int i = i_lo; i < i_hi; ++i) {
        const int buf = (i - i_lo) & 1;
        const int nst = slab_steps(i);
        const int i_next = min(i + 1, i_hi - 1);               // the last slab fetches itself again, unused
        const int byte0_next = slab_byte0(i_next);
        // The next slab's pieces are fetched after this slab's first step (that buffer's last readers passed the barrier
        // long ago): the loop's first instructions wait for registers that old loads may still target, and a fetch issued
        // in front of them would be waited for as well, a memory round trip per slab.
        const char* xb = lds + buf * PF_SLAB_BYTES + lane * 16;
        auto frag = [&](int s, int j, int p) {
            return *reinterpret_cast<const u32x4*>(xb + ((p * 4 + j) * PF_SPS + s) * PF_FRAG_BYTES);
        };
        // every accumulator sees its three pieces in order; neighbours in the instruction stream are independent
        auto multiply = [&](int s, int j, const u32x4 (&x3)[3]) {
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, wa[t][s]), __builtin_bit_cast(bf16x8, x3[p]), acc[t][j], 0, 0, 0);
        };
        // Straight-line code for every slab: the B operands of a (step, column tile) are read from LDS while the previous
        // one is multiplied (read and used back to back, their latency showed in every group of instructions).  A step
        // that the slab does not have (the ragged end of a row) is multiplied with weights of zero: it adds +-0 to sums
        // that started at +0, which changes no bit -- the decode kernels multiply such a step by a block of zeros.
        u32x4 cur[3], nxt[3];
#pragma unroll
        for (int p = 0; p < 3; ++p) cur[p] = frag(0, 0, p);
#pragma unroll
        for (int s = 0; s < PF_SPS; ++s) {
            if (s >= nst) {   // uniform; rare
#pragma unroll
                for (int t = 0; t < NT; ++t) wa[t][s] = u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int j = 0; j < JT; ++j) {
                const int g = s * JT + j + 1;
                if (g < JT * PF_SPS) {
#pragma unroll
                    for (int p = 0; p < 3; ++p) nxt[p] = frag(g / JT, g % JT, p);
                }
                __builtin_amdgcn_sched_barrier(0);   // the reads stay in front of the instructions that hide them
                multiply(s, j, cur);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int p = 0; p < 3; ++p) cur[p] = nxt[p];
            }
            load_weight_step(byte0_next, s);              // this step's registers are free: the next slab's weights
            if (s == 0) fetch_slab(i_next, buf ^ 1);
        }
        if ((i + 1) % nblk == 0) {   // the share's partial sums are complete
            const int p = i / nblk;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int j = 0; j < JT; ++j) {
                    if (PARTIAL) {
                        const int tile = t0 + t, m = m0 + j * 16 + r16;
                        if (tile < a.n_tiles && m < a.M)
                            *reinterpret_cast<f32x4*>(a.part + (size_t)p * a.part_arr + (size_t)m * a.part_ld + tile * 16 + gq * 4) = acc[t][j];
                    } else {     // added in share order
                        f32x4& T = total[PARTIAL ? 0 : t][PARTIAL ? 0 : j];
                        T.x = add_rn(T.x, acc[t][j].x); T.y = add_rn(T.y, acc[t][j].y);
                        T.z = add_rn(T.z, acc[t][j].z); T.w = add_rn(T.w, acc[t][j].w);
                    }
                    acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
        }
        // the next slab has landed once at most the weight loads issued after it (three steps') are still on their way
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NT * (PF_SPS - 1)) : "memory");
        __syncthreads();
    }
    if (PARTIAL) return;

    // ---- epilogue.  Lane l holds, per tile, prompt row (column) l % 16 and output rows 4 * (l / 16) .. + 3 of the tile.
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tile = t0 + t;
        if (tile >= a.n_tiles) continue;
#pragma unroll
        for (int j = 0; j < JT; ++j) {
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
                    *reinterpret_cast<u32x2*>(reinterpret_cast<char*>(a.xs_out + p * a.xs_out_piece) +
                                              pf_xs_off(m, u >> 3, a.L.F) + (u & 4) * 2) = u32x2{piece[p].x, piece[p].y};
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

// ---- QKV dealt by shares (short prompts: a panel of a few dozen rows is bound by the read of the weights and needs
// more workgroups than the projection's 96 tile groups give): the GEMM leaves the 8 partial sums of every output in
// part, this kernel adds them in share order and runs the projection's epilogue -- the same operations as the GEMM's
// own. ------------------------------------------------------------------------------------------------------------------
__device__ __forceinline__ float pf_share_sum(const float* part, size_t part_arr, size_t at) {
    float t = 0.f;
#pragma unroll
    for (int p = 0; p < PF_NSHARE; ++p) t = add_rn(t, part[(size_t)p * part_arr + at]);
    return t;
}
// one thread per (prompt row, tile, rotary pair): rows pr and pr + 8 of the tile
__global__ __launch_bounds__(256) void k_pf_finish_qkv(PfGemm a) {
    const int hd = a.L.hd, H = a.L.H, Hkv = a.L.Hkv, half = hd >> 1, tph = hd >> 4;
    const int n = a.M * a.n_tiles * 8;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += gridDim.x * blockDim.x) {
        const int pr = idx & 7, tile = (idx >> 3) % a.n_tiles, m = (idx >> 3) / a.n_tiles;
        const size_t at = (size_t)m * a.part_ld + tile * 16 + pr;
        const float rsm = a.rs[m];
        float lo = mul_rn(pf_share_sum(a.part, a.part_arr, at), rsm), hi = mul_rn(pf_share_sum(a.part, a.part_arr, at + 8), rsm);
        const int hs = tile / tph, i = (tile - hs * tph) * 8 + pr, pos = a.pos0 + m;
        if (hs < H + Hkv) rotary_pair(lo, hi, a.cosT[(size_t)pos * half + i], a.sinT[(size_t)pos * half + i]);
        if (hs < H) {
            float* o = a.q + (size_t)m * H * hd + (size_t)hs * hd + i;
            o[0] = lo; o[half] = hi;
        } else {
            const bool isk = hs < H + Hkv;
            const int kvh = isk ? hs - H : hs - H - Hkv;
            bf16_t* o = (isk ? a.kc : a.vc) + ((size_t)kvh * a.L.max_seq + pos) * hd + i;
            o[0] = f32_to_bf16(lo); o[half] = f32_to_bf16(hi);
        }
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
// LONGCTX: the panel ends beyond 8 attention splits (1024 positions); see attn_split (the instance for shorter prompts
// is 5 % faster without that code)
template <int LPP, bool LONGCTX>
__global__ __launch_bounds__(WG_THREADS, 4) void k_pf_attn(PfAttn a) {   // 4 waves per SIMD: two workgroups per compute unit (three: spills, slower)
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
            attn_split<bf16_t, LPP, 0, true, LONGCTX>(a.kc, a.vc, aa, reinterpret_cast<float*>(lds), split, g);
            __syncthreads();
        }
    }
}

}  // namespace sdfp
