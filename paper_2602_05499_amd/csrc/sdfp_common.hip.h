// Device code of libsdfp for gfx950 (CDNA4, wave64): the phases of one transformer forward of M <= 16 rows
// over a contiguous KV cache, plus the token-selection kernels of the speculative step
// (paper Sec. II-A Eq. 1-3, Alg. 1 Stage B).
//
// Precision contract: weight matrices and KV entries are stored as float32 or bfloat16; every activation,
// accumulator and logit is float32.  Every output row's arithmetic (order of every sum) is independent of
// how many rows M share the launch, so row i of a (K+1)-row verify forward is bit-identical to the one-row
// decode of the same prefix: this is what makes greedy speculative output equal plain decoding exactly.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sdfp {

typedef unsigned short bf16_t;   // raw bfloat16 bits
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int MAX_K = 8;
constexpr int MAX_ROWS = 16;      // rows of one forward: K + 1 <= 9 for verify, 16 per prompt chunk
constexpr int WG_THREADS = 512;  // every forward-pass kernel runs 8 waves per workgroup, one workgroup per CU
constexpr int NWAVE = WG_THREADS / 64;
constexpr int ATT_SL = 128;      // attention split length in positions (fixed absolute boundaries)
constexpr int ATT_QC = 16;       // query vectors processed per pass inside an attention workgroup

// Pointers read from descriptors in memory have no known address space; without these casts the compiler
// emits FLAT accesses (which also occupy the LDS counter) and vector loads for wave-uniform descriptor reads.
#define SDFP_GLOBAL __attribute__((address_space(1)))
#define SDFP_CONST __attribute__((address_space(4)))
template <class T>
__device__ __forceinline__ SDFP_GLOBAL T* as_global(T* p) {
    return (SDFP_GLOBAL T*)p;
}
template <class T>
__device__ __forceinline__ const SDFP_CONST T* as_const(const T* p) {   // memory nobody writes during the launch
    return (const SDFP_CONST T*)p;
}

// ---- optional guard build (-DSDFP_GUARD): every global access of the forward kernel is checked against the
// ranges of the workspace, the KV buffer and the weights; an access outside them is skipped and recorded, so
// the guarded kernel cannot fault on a bad address.  The product build compiles the checks away.
struct GuardRanges {
    const char* lo[3];
    const char* hi[3];
    unsigned long long* rec;   // rec[0] = violations; then (site, address, bytes | wg << 32) of the first 10
    unsigned* beacon;          // [n_wg][8 waves][2] progress codes (pinned host memory), or nullptr
    unsigned long long* probe; // [n_wg][8 waves][PROBE_N] addresses of the first weight loads of lane 0 (probe build)
    const void* prog;          // the phase list and its length, to bound the descriptor walk
    int prog_len, pad_;
};
constexpr int PROBE_N = 48;
#ifdef SDFP_GUARD
__shared__ GuardRanges s_guard;
__device__ __noinline__ bool guard_fail(const void* p, int bytes, int site) {
    unsigned long long* rec = s_guard.rec;
    const unsigned long long n = __hip_atomic_fetch_add(rec, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    if (n < 10) {
        __hip_atomic_store(rec + 1 + 3 * n, (unsigned long long)site, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(rec + 2 + 3 * n, (unsigned long long)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(rec + 3 + 3 * n, (unsigned long long)(unsigned)bytes | ((unsigned long long)blockIdx.x << 32) |
                           ((unsigned long long)threadIdx.x << 48), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    return false;
}
__device__ __forceinline__ bool guard_ok(const void* p, int bytes, int site) {
    const char* c = (const char*)p;
#pragma unroll
    for (int i = 0; i < 3; ++i)
        if (c >= s_guard.lo[i] && c + bytes <= s_guard.hi[i]) return true;
    return guard_fail(p, bytes, site);
}
__device__ __forceinline__ bool guard_in(const void* p, int bytes, const void* lo, const void* hi, int site) {
    const char* c = (const char*)p;
    if (c >= (const char*)lo && c + bytes <= (const char*)hi) return true;
    return guard_fail(p, bytes, site);
}
// progress code of this wave, written through to host memory
__device__ __forceinline__ void beacon(unsigned code, int slot = 0) {
    if (s_guard.beacon != nullptr && (threadIdx.x & 63) == 0) {
        __hip_atomic_store(s_guard.beacon + (blockIdx.x * 8 + (threadIdx.x >> 6)) * 2 + slot, code, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
}
#define SDFP_OK(p, bytes, site) guard_ok((const void*)(p), (bytes), (site))
#define SDFP_IN(p, bytes, lo, hi, site) guard_in((const void*)(p), (bytes), (lo), (hi), (site))
#define SDFP_BEACON(code) beacon(code)
#define SDFP_BEACON2(code) beacon(code, 1)
#else
#define SDFP_OK(p, bytes, site) true
#define SDFP_IN(p, bytes, lo, hi, site) true
#define SDFP_BEACON(code) ((void)0)
#define SDFP_BEACON2(code) ((void)0)
#endif

// streaming (read-once) 16-byte weight load
__device__ __forceinline__ u32x4 ld_stream(const void* p, const void* lo, const void* hi) {
    if (!SDFP_IN(p, 16, lo, hi, 8)) return u32x4{0u, 0u, 0u, 0u};
#ifdef SDFP_PROBE
    return u32x4{0u, 0u, 0u, 0u};   // the probe build performs no weight load (the loader records the address)
#endif
    // A plain (not non-temporal) load on purpose: a wave's consecutive steps cover the two halves of each
    // 128-byte line with separate instructions, and a non-temporal line is not kept for the second one.
    return *(const SDFP_GLOBAL u32x4*)p;
}
__device__ __forceinline__ f32x4 ld_g4(const float* p) {   // plain 16-byte global load
    if (!SDFP_OK(p, 16, 9)) return f32x4{0.f, 0.f, 0.f, 0.f};
    return *(const SDFP_GLOBAL f32x4*)p;
}
__device__ __forceinline__ float ld_g(const float* p) {
    if (!SDFP_OK(p, 4, 10)) return 0.f;
    return *(const SDFP_GLOBAL float*)p;
}
__device__ __forceinline__ int ld_gi(const int* p) {
    if (!SDFP_OK(p, 4, 11)) return 0;
    return *(const SDFP_GLOBAL int*)p;
}
__device__ __forceinline__ unsigned atomic_inc_g(unsigned* p) {   // returning agent-scope add of 1
    if (!SDFP_OK(p, 4, 12)) return 0u;
    return atomicAdd(p, 1u);
}

// ---- device-resident decode state: written by kernels, read by the next call without host round trips ---
struct DevState {
    int P;          // cache_len: positions held in the KV cache
    int t_last;     // pending token
    int n_acc;      // accepted draft tokens of the last step
    int x;          // extra target-derived token of the last step
    int K;          // speculation depth of the current step
    int n_out;      // committed tokens in the output list
    int max_out;
    int overflow;   // set if the output list was full
    long long steps, drafted, accepted, examined;
    int d[MAX_K];           // draft block
    int amax[MAX_ROWS];     // arg-max of each verify row
};

// Which tokens / positions the rows of a forward hold.
enum { ROWS_PROMPT = 0, ROWS_DRAFT = 1, ROWS_VERIFY = 2 };
struct Rows {
    int M;     // number of rows
    int src;   // ROWS_*
    int off;   // ROWS_PROMPT: absolute position of row 0; ROWS_DRAFT: draft index i (row sits at P + i)
};

__device__ __forceinline__ int row_pos(const Rows& r, const DevState* st, int m) {
    if (r.src == ROWS_PROMPT) return r.off + m;
    if (r.src == ROWS_DRAFT) return ld_gi(&st->P) + r.off;
    return ld_gi(&st->P) + m;
}
__device__ __forceinline__ int row_tok(const Rows& r, const DevState* st, const int* prompt, int m) {
    if (r.src == ROWS_PROMPT) return ld_gi(prompt + r.off + m);
    int i = (r.src == ROWS_DRAFT) ? r.off : m;
    return i == 0 ? ld_gi(&st->t_last) : ld_gi(&st->d[i - 1]);
}

// ---- agent-coherent accesses ------------------------------------------------------------------------------
// Data that one workgroup writes and another reads INSIDE one kernel (activations, new KV rows, partials)
// goes through relaxed agent-scope atomics: the hardware marks such loads/stores device-coherent (sc1), so
// they are visible across the eight XCDs' L2 caches as soon as the store is acknowledged.  This lets the
// grid barrier and the last-arriver reductions work without whole-cache write-back / invalidate fences.
__device__ __forceinline__ float ld_coh(const float* p) {
    if (!SDFP_OK(p, 4, 1)) return 0.f;
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_coh(const int* p) {
    if (!SDFP_OK(p, 4, 2)) return 0;
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u32x2 ld_coh8(const void* p) {   // 8-byte aligned
    const unsigned long long v = __hip_atomic_load(as_global(reinterpret_cast<const unsigned long long*>(p)), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    return u32x2{(unsigned)v, (unsigned)(v >> 32)};
}
__device__ __forceinline__ f32x4 ld_coh4(const float* p) {  // 16-byte aligned
    const u32x2 a = ld_coh8(p), b = ld_coh8(p + 2);
    return f32x4{__uint_as_float(a.x), __uint_as_float(a.y), __uint_as_float(b.x), __uint_as_float(b.y)};
}
// loads of activations that another workgroup wrote earlier in this launch
#ifdef SDFP_COH_ACT
__device__ __forceinline__ f32x4 ld_act4(const float* p) { return ld_coh4(p); }
__device__ __forceinline__ float ld_act(const float* p) { return ld_coh(p); }
__device__ __forceinline__ u32x2 ld_act8(const void* p) { return ld_coh8(p); }
#else
__device__ __forceinline__ f32x4 ld_act4(const float* p) { return ld_g4(p); }
__device__ __forceinline__ float ld_act(const float* p) { return ld_g(p); }
__device__ __forceinline__ u32x2 ld_act8(const void* p) {
    if (!SDFP_OK(p, 8, 20)) return u32x2{0u, 0u};
    return *(const SDFP_GLOBAL u32x2*)p;
}
#endif
__device__ __forceinline__ void st_coh(float* p, float v) {
    if (!SDFP_OK(p, 4, 3)) return;
    __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coh(int* p, int v) {
    if (!SDFP_OK(p, 4, 4)) return;
    __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coh(unsigned* p, unsigned v) {
    if (!SDFP_OK(p, 4, 5)) return;
    __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coh(bf16_t* p, bf16_t v) {
    if (!SDFP_OK(p, 2, 6)) return;
    __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coh4(float* p, const f32x4& v) {   // 16-byte aligned
    if (!SDFP_OK(p, 16, 7)) return;
    SDFP_GLOBAL unsigned long long* q = as_global(reinterpret_cast<unsigned long long*>(p));
    __hip_atomic_store(q, (unsigned long long)__float_as_uint(v.x) | ((unsigned long long)__float_as_uint(v.y) << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(q + 1, (unsigned long long)__float_as_uint(v.z) | ((unsigned long long)__float_as_uint(v.w) << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// grid-barrier words in the workspace: bar[0] global count, bar[BAR_FLAG_OFF] sticky time-out flag,
// bar[BAR_STRIDE * (2 + g)] counter of group g
constexpr int BAR_GROUPS = 8;
constexpr int BAR_STRIDE = 16;                          // unsigneds between counters (64-byte lines)
constexpr int BAR_WORDS = BAR_STRIDE * (BAR_GROUPS + 2);
constexpr int BAR_FLAG_OFF = BAR_STRIDE;

// Hand-over of activations by the data itself: the buffers that one phase writes and the next projection reads are
// pre-armed with this bit pattern at the start of a forward, are written once, and a reader polls until none of
// its values still holds it.  It is a NaN that arithmetic does not produce (hardware makes the canonical quiet NaN);
// only a NaN with this very payload in the caller's weights could imitate it, and then the bounded wait ends the
// forward with the time-out flag instead of a result.
constexpr unsigned HANDOVER_ARMED = 0xFFFFFFFFu;
__device__ __forceinline__ bool armed8(const f32x4& a, const f32x4& b) {   // any of the 8 values not written yet
    const unsigned m0 = max(max(__float_as_uint(a.x), __float_as_uint(a.y)), max(__float_as_uint(a.z), __float_as_uint(a.w)));
    const unsigned m1 = max(max(__float_as_uint(b.x), __float_as_uint(b.y)), max(__float_as_uint(b.z), __float_as_uint(b.w)));
    return max(m0, m1) == HANDOVER_ARMED;
}

// Wait until every store this wave has issued is acknowledged.  A wave calls this before the workgroup
// barrier that precedes signalling other workgroups (the workgroup-scope barrier alone does not wait for
// outstanding vector-memory stores).
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---- storage types -------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((unsigned)b) << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {   // round-to-nearest-even, finite inputs
    unsigned u = __float_as_uint(f);
    return (bf16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
template <typename WT> struct ST;
template <> struct ST<float> {
    static constexpr int VEC = 4;   // elements per 16-byte load
    static __device__ __forceinline__ float ld(const float* p) { return ld_g(p); }
    static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
    static __device__ __forceinline__ void stc(float* p, float v) { st_coh(p, v); }
    static __device__ __forceinline__ void unpack(const u32x4& r, float (&w)[4]) {
        w[0] = __uint_as_float(r.x); w[1] = __uint_as_float(r.y);
        w[2] = __uint_as_float(r.z); w[3] = __uint_as_float(r.w);
    }
};
template <> struct ST<bf16_t> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float ld(const bf16_t* p) {
        if (!SDFP_OK(p, 2, 13)) return 0.f;
        return bf16_to_f32(*(const SDFP_GLOBAL bf16_t*)p);
    }
    static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
    static __device__ __forceinline__ void stc(bf16_t* p, float v) { st_coh(p, f32_to_bf16(v)); }
    static __device__ __forceinline__ void unpack(const u32x4& r, float (&w)[8]) {
        w[0] = __uint_as_float(r.x << 16); w[1] = __uint_as_float(r.x & 0xFFFF0000u);
        w[2] = __uint_as_float(r.y << 16); w[3] = __uint_as_float(r.y & 0xFFFF0000u);
        w[4] = __uint_as_float(r.z << 16); w[5] = __uint_as_float(r.z & 0xFFFF0000u);
        w[6] = __uint_as_float(r.w << 16); w[7] = __uint_as_float(r.w & 0xFFFF0000u);
    }
};

// ---- wave64 reductions on the DPP network (no LDS traffic).  The total lands in the LAST lane of each
// group of G consecutive lanes (G a power of two, 2..64); the summation tree is fixed. -------------------
template <int CTRL, int ROWMASK>
__device__ __forceinline__ float dpp_add(float v) {
    return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWMASK,
                                                                      0xf, false));
}
template <int G>
__device__ __forceinline__ float group_sum_dpp(float v) {
    if (G >= 2) v = dpp_add<0x111, 0xf>(v);    // row_shr:1
    if (G >= 4) v = dpp_add<0x112, 0xf>(v);    // row_shr:2
    if (G >= 8) v = dpp_add<0x114, 0xf>(v);    // row_shr:4
    if (G >= 16) v = dpp_add<0x118, 0xf>(v);   // row_shr:8
    if (G >= 32) v = dpp_add<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    if (G >= 64) v = dpp_add<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ __forceinline__ float wave_sum_last(float v) { return group_sum_dpp<64>(v); }   // valid in lane 63

__device__ __forceinline__ float wave_sum(float v) {   // butterfly: total in every lane
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

struct LayerDims {
    int d, H, Hkv, hd, F, V, max_seq;
};

// ---- arithmetic that several kernels must reproduce bit for bit (one-row decode, verify rows, prompt chunks and the
// prompt's matrix-matrix path all write the same cache and feed the same residual stream).  Every operation is one
// of the primitives below: a single correctly rounded float32 instruction that the compiler may not fuse with its
// neighbours (contraction is switched off inside each, and an operation loses the permission to be fused when either
// side lacks it), so no compiler decision about contraction can differ from one kernel to the next. -------------------
__device__ __forceinline__ float add_rn(float a, float b) {
#pragma clang fp contract(off)
    return a + b;
}
__device__ __forceinline__ float sub_rn(float a, float b) {
#pragma clang fp contract(off)
    return a - b;
}
__device__ __forceinline__ float mul_rn(float a, float b) {
#pragma clang fp contract(off)
    return a * b;
}
__device__ __forceinline__ float fma_rn(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ float div_rn(float a, float b) {   // correctly rounded division
#pragma clang fp contract(off)
    return a / b;
}
__device__ __forceinline__ float sqrt_rn(float a) { return __fsqrt_rn(a); }
// squares of 8 consecutive values, added in one fixed order wherever a row's sum of squares is formed
__device__ __forceinline__ float sq8(const f32x4& a, const f32x4& b) {
    float s = mul_rn(a.x, a.x);
    s = fma_rn(a.y, a.y, s); s = fma_rn(a.z, a.z, s); s = fma_rn(a.w, a.w, s);
    s = fma_rn(b.x, b.x, s); s = fma_rn(b.y, b.y, s); s = fma_rn(b.z, b.z, s); s = fma_rn(b.w, b.w, s);
    return s;
}
// reciprocal root mean square of a row of n values with sum of squares ss (RMSNorm)
__device__ __forceinline__ float rms_recip(float ss, int n, float eps) {
    return div_rn(1.0f, sqrt_rn(add_rn(div_rn(ss, (float)n), eps)));
}
// rotary embedding of one pair: (a, b) -> (a cos - b sin, b cos + a sin)
__device__ __forceinline__ void rotary_pair(float& a, float& b, float c, float sn) {
    const float ra = fma_rn(a, c, -mul_rn(b, sn)), rb = fma_rn(b, c, mul_rn(a, sn));
    a = ra; b = rb;
}
// SwiGLU: silu(gate) * up
__device__ __forceinline__ float swiglu(float gate, float up) {
    return mul_rn(div_rn(gate, add_rn(1.0f, __expf(-gate))), up);
}
// A float32 activation as three bfloat16 pieces x = x0 + x1 + x2, each the round-to-nearest-even bfloat16 of what the
// previous ones left (every remainder is exact in float32): 8 values -> three packed quads, value k in half k % 2 of
// word k / 2.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));   // the matrix-core bf16 operand of one lane
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16(float a, float b) {   // round-to-nearest-even pair, a in the low half
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}
// emit(s, quad) is called for piece s = 0, 1, 2 as soon as it exists, so that a caller that stores each piece at once
// keeps one quad alive, not three
template <class Emit>
__device__ __forceinline__ void split3_bf16_each(const float (&x)[8], Emit emit) {
    float r[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = x[e];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        u32x4 pk;
        pk.x = pack_bf16(r[0], r[1]); pk.y = pack_bf16(r[2], r[3]);
        pk.z = pack_bf16(r[4], r[5]); pk.w = pack_bf16(r[6], r[7]);
        emit(s, pk);
        if (s + 1 < 3) {   // the remainder is exact in float32
            r[0] = sub_rn(r[0], __uint_as_float(pk.x << 16)); r[1] = sub_rn(r[1], __uint_as_float(pk.x & 0xFFFF0000u));
            r[2] = sub_rn(r[2], __uint_as_float(pk.y << 16)); r[3] = sub_rn(r[3], __uint_as_float(pk.y & 0xFFFF0000u));
            r[4] = sub_rn(r[4], __uint_as_float(pk.z << 16)); r[5] = sub_rn(r[5], __uint_as_float(pk.z & 0xFFFF0000u));
            r[6] = sub_rn(r[6], __uint_as_float(pk.w << 16)); r[7] = sub_rn(r[7], __uint_as_float(pk.w & 0xFFFF0000u));
        }
    }
}
__device__ __forceinline__ void split3_bf16(const float (&x)[8], u32x4 (&piece)[3]) {
    split3_bf16_each(x, [&](int s, const u32x4& pk) { piece[s] = pk; });
}

}  // namespace sdfp
