/* sdfp.h -- C-ABI of libsdfp: the speculative draft-and-verify decode step on one MI355X (gfx950).
 *
 * The method (paper Sec. II-A, Alg. 1 Stage B, Sec. III-C): a draft model -- the target transformer with
 * the layers of a given prune set removed, sharing the target's weights and KV cache -- proposes K tokens
 * one after another (Eq. 1); the full model scores the K proposals in one causal (K+1)-row forward; an
 * accept/reject rule (Eq. 2) commits the longest accepted prefix plus one target-derived token (Eq. 3 on
 * rejection); the KV cache is rolled back to the committed length.  The prune set (Alg. 1 Stage A) is an
 * input here: a per-layer skip mask.
 *
 * Conventions
 *  - Every pointer is marked HOST or DEVICE.  The caller owns all device memory (weights, KV buffer,
 *    workspace) and the HIP stream; the library borrows them until sd_free, never allocates device memory
 *    and never copies or repacks weights: draft and target read the same buffers.
 *  - Weight matrices are row-major [out_features][in_features] in the storage type `dtype` (float32 or
 *    bfloat16); RMSNorm gains are float32.  The KV cache uses the same storage type; all activations,
 *    logits and accumulations are float32.
 *  - sd_draft / sd_verify / sd_accept / sd_rollback / sd_decode only enqueue work on the stream and return;
 *    token ids, the accepted count and the cache length stay in device memory and feed the next call.
 *    sd_prefill waits for the stream once, after the prompt has been copied to the device (so that
 *    prompt_host may be reused on return), and again during the first call on a context (upload of the
 *    rotary table and the phase lists); the forwards it enqueues afterwards are not waited for.  Besides it
 *    only sd_read, sd_dump_*, sd_sync, the diagnostics' *_read calls, and sd_set_skip_mask once a context has
 *    run wait for the stream.
 *  - Every function returns 0 (SD_OK) or a negative SD_E* code; argument, state and capacity errors are
 *    detected on the host before anything is enqueued.  No exceptions, no aborts.
 *  - Call order: sd_init -> sd_prefill -> { sd_draft -> sd_verify -> sd_accept -> sd_rollback }* or
 *    { sd_decode }*.  Between steps the cache holds the keys/values of every committed token except the
 *    last one, which is pending (it is the first input of the next step).
 *  - A context is not thread-safe; calls on one context must come from one thread at a time.
 */
#ifndef SDFP_H
#define SDFP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sd_ctx sd_ctx; /* opaque */

enum { SD_F32 = 0, SD_BF16 = 1 };                 /* storage type of weight matrices and KV cache        */
enum { SD_GREEDY = 0, SD_SAMPLE = 1 };            /* decoding mode                                       */
enum { SD_LOGITS_DRAFT = 0, SD_LOGITS_VERIFY = 1 };
enum { SD_SKIP_ATTN = 1, SD_SKIP_FFN = 2 };       /* skip-mask bits per layer (3 = whole layer)          */
enum {
    SD_OK = 0,
    SD_EINVAL = -1,    /* null pointer, bad size, bad dtype/mode, K out of range                         */
    SD_ECAPACITY = -2, /* prompt or cache_len + K + 1 exceeds max_seq, or output list full               */
    SD_ESTATE = -3,    /* call out of order                                                              */
    SD_EHIP = -4,      /* a HIP call failed; sd_last_hip_error gives its code                            */
    SD_ENOMEM = -5,    /* kv_bytes / ws_bytes smaller than sd_kv_bytes / sd_workspace_bytes              */
    SD_ETIMEOUT = -6   /* a bounded wait inside the forward kernel expired (reported by sd_read); the      */
                       /* results of that forward are invalid                                            */
};
#define SD_MAX_K 8     /* largest speculation depth supported (verify forward has at most 9 rows)        */

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t max_seq;     /* KV capacity in positions; a step needs cache_len + K + 1 <= max_seq           */
    int32_t max_k;       /* largest K any sd_draft call will use, 0..SD_MAX_K                            */
    int32_t dtype;       /* SD_F32 | SD_BF16                                                             */
    int32_t max_out;     /* capacity of the device-side list of committed tokens                        */
    float rms_eps;       /* RMSNorm epsilon                                                              */
    float rope_theta;    /* rotary base; pairs (i, i + head_dim/2), angle = pos * theta^(-2i/head_dim)    */
    float temperature;   /* soft-max temperature for SD_SAMPLE (> 0); ignored when greedy                */
} sd_config;

/* All tensor pointers are DEVICE pointers; the nine per-layer arrays are HOST arrays of n_layers DEVICE
 * pointers.  Shapes: tok_emb, lm_head [vocab][d_model]; wq [n_heads*head_dim][d_model]; wk, wv
 * [n_kv_heads*head_dim][d_model]; wo [d_model][n_heads*head_dim]; w_gate, w_up [d_ffn][d_model];
 * w_down [d_model][d_ffn]; norms [d_model] float32. */
typedef struct {
    const void *tok_emb;
    const float *final_norm;
    const void *lm_head;
    const float *const *attn_norm;
    const void *const *wq, *const *wk, *const *wv, *const *wo;
    const float *const *ffn_norm;
    const void *const *w_gate, *const *w_up, *const *w_down;
} sd_weights;

typedef struct {
    int64_t steps;     /* draft/verify/accept steps taken                                                */
    int64_t drafted;   /* draft tokens proposed (K per step)                                             */
    int64_t accepted;  /* draft tokens accepted                                                          */
    int64_t examined;  /* draft tokens examined before the step's decision: n + [n < K]                  */
    int64_t committed; /* tokens committed so far, including the prefill's first token                   */
    int32_t cache_len; /* positions held in the KV cache                                                 */
    int32_t t_last;    /* pending token                                                                  */
    int32_t last_n;    /* accepted count of the most recent step                                         */
    int32_t last_k;    /* speculation depth of the most recent step                                      */
} sd_stats;

/* Bytes the caller must provide for the KV cache ([layer][K|V][kv_head][max_seq][head_dim] in the storage
 * type) and for the workspace (activations, attention partials, logits rows, rotary table, device state, and for
 * bfloat16 storage the buffers of a panel of up to 512 prompt rows of the matrix-matrix prompt path, at most 1 GiB).
 * Return 0 if the configuration is invalid. */
size_t sd_kv_bytes(const sd_config *cfg);
size_t sd_workspace_bytes(const sd_config *cfg);

/* Create a context.  cfg, w, skip_mask: HOST (copied).  skip_mask[n_layers]: the prune set of Alg. 1
 * Stage A as SD_SKIP_* bits; NULL means no layer is skipped.  kv_buf, ws_buf: DEVICE, 256-byte aligned,
 * at least sd_kv_bytes / sd_workspace_bytes long, owned by the caller and borrowed until sd_free.
 * hip_stream: a hipStream_t (NULL = the default stream).  Performs no GPU work.  The forward kernels run one
 * workgroup per compute unit and need all of them resident at once; the first launch of each kernel checks
 * that a workgroup fits on a compute unit and returns SD_EINVAL from that call if it does not. */
int sd_init(sd_ctx **out, const sd_config *cfg, const sd_weights *w, const uint8_t *skip_mask, void *kv_buf,
            size_t kv_bytes, void *ws_buf, size_t ws_bytes, void *hip_stream);

/* For callers that cannot allocate device memory (set-up code around HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): sd_init without a workspace argument.  The workspace is an array of
 * SD_STATIC_WS_BYTES that is part of the library image on every GPU the library runs on (held until the process
 * ends); the context itself lives in static host storage.  The call allocates nothing, on the device or on the
 * host, and performs no GPU work; its first call on a device looks up where that device's copy of the array lives
 * (the device must be current, as for every call on the context).  The array holds the compact form of the
 * workspace: what sd_workspace_bytes counts, less the room it adds for a full 512-row panel of the matrix-matrix
 * prompt path (long prompts then go through smaller panels, or through 16-row chunks; same results).
 * Configurations whose compact workspace exceeds SD_STATIC_WS_BYTES (the 7B benchmark shape fits; 13B and wider
 * shapes do not) or that have more than SD_STATIC_MAX_LAYERS layers are refused with SD_ENOMEM.  All such
 * contexts of one GPU would share the one array, so there is one at a time per GPU: a second call before sd_free
 * of the first returns SD_ESTATE.  The array keeps what the previous context left; the first sd_prefill clears
 * what must start at zero, as it does for a caller's workspace.  Everything else -- arguments, results, errors,
 * the calls that follow -- is as for sd_init; the context computes bit-identical results. */
#define SD_STATIC_WS_BYTES (64u << 20)
#define SD_STATIC_MAX_LAYERS 128
int sd_init_static(sd_ctx **out, const sd_config *cfg, const sd_weights *w, const uint8_t *skip_mask, void *kv_buf,
                   size_t kv_bytes, void *hip_stream);

/* Replace the prune set (HOST uint8[n_layers], copied).  Takes effect from the next sd_draft. */
int sd_set_skip_mask(sd_ctx *ctx, const uint8_t *skip_mask);

/* Target forward over the prompt ("given input x", Sec. II-A): fills the KV cache for positions 0..n-1 in
 * every layer, picks the first generated token from the last row (arg-max, or inverse-CDF sampling with
 * u_host[0]) and commits it; cache_len = n.  prompt_host: HOST int32[n], 1 <= n, n + max_k + 1 <= max_seq.
 * u_host: HOST float[1] in [0,1) when mode == SD_SAMPLE, else ignored (may be NULL).  Resets the output
 * list and the statistics. */
int sd_prefill(sd_ctx *ctx, const int32_t *prompt_host, int32_t n, int mode, const float *u_host);

/* Eq. 1: K autoregressive one-row forwards of the layer-skipped model starting from the pending token,
 * at positions cache_len..cache_len+K-1, reading the shared cache and writing K/V only for layers that
 * run.  Draft tokens are arg-maxes (greedy) or inverse-CDF samples with u_host[0..K-1] (HOST, sampling).
 * 0 <= K <= max_k; cache_len + K + 1 <= max_seq or SD_ECAPACITY. */
int sd_draft(sd_ctx *ctx, int32_t K, int mode, const float *u_host);

/* Target evaluation of the proposed block (the operands of Eq. 2): one causal (K+1)-row forward of the
 * full model over [pending, d_1..d_K] at positions cache_len..cache_len+K; overwrites the cache at those
 * positions in every layer; leaves K+1 logits rows (and their arg-maxes) in the workspace. */
int sd_verify(sd_ctx *ctx);

/* Eq. 2 / Eq. 3: n = number of accepted draft tokens, x = the extra target-derived token; appends
 * d_1..d_n, x to the device-side output list and updates the statistics.  Greedy: accept while d_{i+1}
 * equals the arg-max of target row i; x = arg-max of row n.  Sampling: accept d_{i+1} iff
 * u_host[i] * q_i(d_{i+1}) < p_i(d_{i+1}); x ~ max(0, p_n - q_n) (normalised) if n < K, x ~ p_K otherwise,
 * drawn by inverse CDF with u_host[K].  u_host: HOST float[K+1] (sampling) or NULL (greedy).
 * mode must equal the mode of the preceding sd_draft. */
int sd_accept(sd_ctx *ctx, int mode, const float *u_host);

/* In-place KV rollback: cache_len += n + 1, pending token = x.  Entries past the new length are dead and
 * are overwritten by the next step; nothing is moved. */
int sd_rollback(sd_ctx *ctx);

/* One step of vanilla autoregressive decoding with the full model (the baseline of Table 1): equivalent
 * to sd_draft(K = 0), sd_verify, sd_accept, sd_rollback.  u_host: HOST float[1] when sampling. */
int sd_decode(sd_ctx *ctx, int mode, const float *u_host);

/* Teacher forcing / resume: overwrite the device-side (cache_len, pending token) pair, e.g. to restart
 * from an earlier committed length, and replace the draft block by d_host[0..K-1] (HOST) so that
 * sd_verify scores an externally proposed block.  Neither touches the KV cache. */
int sd_set_pending(sd_ctx *ctx, int32_t cache_len, int32_t token);
int sd_set_draft(sd_ctx *ctx, const int32_t *d_host, int32_t K);

/* Wait for the stream, then copy out up to cap committed tokens (HOST int32, may be NULL with cap 0), the
 * number committed (may be NULL) and the statistics (may be NULL). */
int sd_read(sd_ctx *ctx, int32_t *tokens_host, int32_t cap, int32_t *n_committed, sd_stats *stats);

/* Wait for the stream and copy logits rows of the most recent draft block ([K][vocab]) or verify forward
 * ([K+1][vocab]) to HOST float memory holding at least `cap` floats; draft tokens to HOST int32[K].
 * For parity tests. */
int sd_dump_logits(sd_ctx *ctx, int which, float *host, size_t cap);
int sd_dump_draft(sd_ctx *ctx, int32_t *d_host, int32_t cap);

/* Enable (1) or disable (0) storing full logits rows in greedy mode (they are always stored when
 * sampling).  Greedy arg-max is fused into the output projection either way. */
int sd_keep_logits(sd_ctx *ctx, int on);

/* Diagnostics.  sd_phase_trace(1) makes every following forward record the timeline of its workgroup 0:
 * one entry per phase body and per phase boundary, (tag << 56) | ticks of the 100 MHz device clock, tag =
 * 2 * phase + {0 body finished, 1 boundary passed: the grid barrier, or only the workgroup's own barrier where
 * the rows go to the next phase by themselves}, phase: 0 start, 1 embedding, 2 QKV, 3 attention,
 * 4 O-projection, 5 gate/up, 6 down, 7 output head, 15 final arg-max reduce.  sd_phase_trace_read waits for the stream and copies the entries
 * of the most recent forward (HOST uint64[cap]); *n receives their number. */
int sd_phase_trace(sd_ctx *ctx, int on);
int sd_phase_trace_read(sd_ctx *ctx, uint64_t *host, int32_t cap, int32_t *n);

/* Bound of every wait inside the forward kernel, in polls (default 2^21, several hundred milliseconds).  When a
 * wait expires the kernel raises a sticky flag, lets every later wait fall through and terminates normally; the
 * results of that forward and of every later one are invalid and sd_read returns SD_ETIMEOUT until the next
 * sd_prefill, which re-arms the barrier state.  A tiny bound lets a test exercise that path.  (Inside a forward
 * a float32 whose bits are 0xFFFFFFFF marks an activation that is not written yet; finite inputs never produce
 * it, but a weight tensor that holds NaNs with that payload can make a forward end this way.) */
int sd_set_spin_limit(sd_ctx *ctx, uint32_t polls);

/* Which set of decode kernels runs (draft, verify, plain decode; prompt chunks have one set).  In one set a turn of
 * the weight ring holds blocks of one 16-row tile; in the other it may go on into the next tile, which pays where
 * the blocks of a weight row do not fill whole turns (e.g. d_model 5120 in bf16: five 2 KB blocks against turns of
 * four) and costs a little elsewhere.  mode: -1 = choose from the shapes (the default), 0 = never, 1 = always.  Both
 * sets compute bit-identical results; the switch exists so that tests can run either on any shape. */
int sd_set_turn_span(sd_ctx *ctx, int mode);

/* How sd_prefill runs the prompt.  0: through the weight-streaming forward kernel, 16 rows at a time (every weight is
 * re-read per 16 rows).  1: as matrix-matrix products on the matrix cores, in panels of up to 512 rows whose buffers
 * live in the workspace's activation region (bfloat16 storage only; SD_EINVAL if the configuration has no room for a
 * panel).  -1 (the default): 1 for bfloat16 prompts of 5 rows or more, else 0.  Both fill the cache, and produce the
 * logits of the last row, bit-identically to each other and to one-row decoding of the same tokens; the switch exists
 * so that tests can run either on any prompt. */
int sd_set_prefill_mode(sd_ctx *ctx, int mode);

/* Optional, for the matrix-matrix prompt forward (Sec. II-A, "given input x"; bfloat16 storage): a second copy of
 * every layer's projection matrices in the order that path reads them -- per 16-row tile and 64-byte step of the
 * reduction dimension one contiguous kilobyte -- so that a step is a few whole cache lines instead of 64 separate
 * 16-byte accesses.  Same results bit for bit; the 512-token prompt of the 7B benchmark shape takes 22 ms with it
 * instead of 27, and the decode-time forwards, which read their O and down projections from it where d_model / 16
 * divides by the number of compute units, 1.5-2 % less (everything else they keep reading from the caller's matrices).
 * sd_tiled_weights_bytes: bytes of the copy (the size of the layer matrices; 0 for float32 storage or a bad cfg).
 * sd_set_tiled_weights: buf is DEVICE memory, 256-byte aligned, owned by the caller and borrowed until sd_free or
 * until the next call of this function; the call enqueues the copy kernels on the context's stream (the weights must
 * be final by then; call it again after changing them).  buf == NULL detaches the copy.  Errors: SD_EINVAL (ctx,
 * alignment, float32 storage), SD_ENOMEM (bytes too small), SD_EHIP. */
size_t sd_tiled_weights_bytes(const sd_config *cfg);
int sd_set_tiled_weights(sd_ctx *ctx, void *buf, size_t bytes);

/* Diagnostics of a library built with -DSDFP_GUARD (every global access of the forward kernel range-checked,
 * bad ones skipped and recorded).  Waits for the stream and copies the record to HOST uint64[32]: [0] number
 * of violations, then (site, address, bytes | workgroup << 32 | thread << 48) of the first ten.  A product
 * build records nothing. */
int sd_guard_read(sd_ctx *ctx, uint64_t *host32);
/* Guard build only: put the record (32 uint64) and, after it, one progress code per workgroup and wave
 * (uint32[1024][8][2]) into PINNED HOST memory owned by the caller, so that they survive a device fault. */
int sd_guard_host_buffer(sd_ctx *ctx, uint64_t *pinned, size_t bytes);

int sd_sync(sd_ctx *ctx);                 /* wait for the stream                                          */
int sd_last_hip_error(const sd_ctx *ctx); /* HIP status behind the last SD_EHIP                           */
void sd_free(sd_ctx *ctx);                /* releases host-side resources only                            */
const char *sd_strerror(int code);

/* ---- Draft construction: FIT layer scores and the prune set (Sec. III-B, Eq. 11; Alg. 1 Stage A) ------------------
 * T_l = 1/N sum_i || grad_{theta_l} f(z_i, theta) ||_2^2 over a calibration set of N token sequences of T tokens each,
 * f = the mean next-token cross-entropy of the sequence (logits at positions 0 .. T-2 against tokens 1 .. T-1), theta_l
 * = the nine tensors of layer l.  The sum is returned in two parts: t_attn[l] for the attention sub-layer (attn_norm,
 * wq, wk, wv, wo) and t_ffn[l] for the feed-forward sub-layer (ffn_norm, w_gate, w_up, w_down); the layer score of
 * Alg. 1 is their sum.  The forward is the whole-sequence forward of the model with float32 activations (weights as
 * stored; keys and values are not rounded, there is no cache), the gradients are exact derivatives of that forward in
 * float32.  cfg: as for sd_init; only bfloat16 storage, T in 2..2048, and d_model, n_heads * head_dim,
 * n_kv_heads * head_dim, d_ffn and vocab multiples of 32 (else SD_EINVAL, and sd_fit_workspace_bytes returns 0);
 * max_seq, max_k, max_out and temperature are ignored.  w: DEVICE pointers in a HOST struct, as for sd_init, read
 * only.  tokens_host: HOST, [n_samples][T].  ws_buf: DEVICE, 256-byte aligned, sd_fit_workspace_bytes(cfg, T) bytes,
 * scratch (about L * (10 T d + 2 T F + H T^2) floats: the activations the backward needs), free for reuse on return; if
 * ws_bytes exceeds that by the bytes of all layer matrices and the output head (rounded up to 256 each) and there is
 * more than one sample, the surplus keeps the transposed matrices of the backward from the first sample on; with as
 * much again, also copies of the matrices in the tile order the forward products read fastest.
 * t_attn_host, t_ffn_host: HOST, [n_layers] each; loss_host: HOST, [n_samples] or NULL, the samples' losses.
 * Needs no context; enqueues on hip_stream and waits for it before returning.  Float32 sums of different order from
 * run to run (atomic adds) make the scores reproducible to about 1e-6 relative, not bit for bit.
 * Errors: SD_EINVAL (arguments, token out of range), SD_ENOMEM (ws_bytes too small), SD_EHIP. */
size_t sd_fit_workspace_bytes(const sd_config *cfg, int32_t T);
int sd_fit_scores(const sd_config *cfg, const sd_weights *w, const int32_t *tokens_host, int32_t n_samples, int32_t T,
                  void *ws_buf, size_t ws_bytes, void *hip_stream, double *t_attn_host, double *t_ffn_host,
                  double *loss_host);
/* Alg. 1 Stage A, last step (host only): mask_out[l] = SD_SKIP_ATTN | SD_SKIP_FFN for the floor(ratio * n_layers)
 * layers of smallest t_attn[l] + t_ffn[l] (equal scores: the lower index first), 0 for the others.  All HOST.
 * Errors: SD_EINVAL (null pointer, n_layers < 1, ratio outside [0, 1]). */
int sd_fit_prune_mask(const double *t_attn, const double *t_ffn, int32_t n_layers, double ratio, uint8_t *mask_out);
/* The same ranking per kind of sub-layer (Sec. IV-A prunes attention and feed-forward sub-layers at separate ratios, e.g.
 * one half of the attention and 35 % of the feed-forward sub-layers of a 13B model): SD_SKIP_ATTN for the
 * floor(ratio_attn * n_layers) layers of smallest t_attn, SD_SKIP_FFN for the floor(ratio_ffn * n_layers) layers of
 * smallest t_ffn, ranked separately.  All HOST; errors as above. */
int sd_fit_prune_sublayers(const double *t_attn, const double *t_ffn, int32_t n_layers, double ratio_attn, double ratio_ffn,
                           uint8_t *mask_out);

#ifdef __cplusplus
}
#endif
#endif /* SDFP_H */
