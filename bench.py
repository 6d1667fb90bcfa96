#!/usr/bin/env python3
"""Benchmark of the speculative draft-and-verify decode step on one MI355X.

A "step" is one pass of the whole hot path: K one-row draft forwards of the layer-skipped model, one
(K+1)-row verify forward of the full model, accept, rollback.  The workload is the Llama-2-7B-shaped
configuration (bf16 storage, 32 layers, 16 skipped by a seeded mask, K=4, greedy, batch 1, 512-token
prompt, generation window of 256 tokens) with seeded random-init weights created directly in HBM.

Prints ONE JSON line: committed tokens/s of speculative decoding (value), of plain autoregressive
decoding through the same kernels, per-step draft / verify latency, achieved HBM GB/s against the 8 TB/s
peak ("roofline"), the prompt forward (matrix-matrix path) against the MFMA peak ("prefill"), the projected
speed-up versus acceptance rate, and the CPU oracle timed on the host cores on a bounded sample of the same
workload ("cpu_baseline").
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


EXTRA_WARMUP_MAX = 400   # most untimed steps that --min-warmup-s may add (buffers are sized for them)


def algorithmic_bytes(s, n_attn, n_ffn, rows, ctx_len):
    """Bytes one forward must move: the weights of the n_attn attention sub-layers and n_ffn FFN sub-layers that
    run and the output head once, the KV cache of those attention sub-layers read once (ctx_len positions) and
    written for `rows` positions, the embedding rows."""
    B = 4 if s.dtype == "f32" else 2
    hq, hk = s.n_heads * s.head_dim, s.n_kv_heads * s.head_dim
    attn_w = (hq * s.d_model + 2 * hk * s.d_model + s.d_model * hq) * B + s.d_model * 4
    ffn_w = 3 * s.d_ffn * s.d_model * B + s.d_model * 4
    head = s.vocab * s.d_model * B + s.d_model * 4
    kv_read = 2 * hk * B * ctx_len
    kv_write = 2 * hk * B * rows
    return n_attn * (attn_w + kv_read + kv_write) + n_ffn * ffn_w + head + rows * s.d_model * B


def prompt_flops(s, n):
    """Multiply-add flops (2 per MAC) of the prompt forward of n tokens as the method defines it: every projection of
    every layer for n rows, causal attention (scores and weighted sum over i + 1 positions for row i), the output
    head for the last row only.  One pass per product: the kernels split each float32 activation into three bfloat16
    pieces and so execute three MFMA passes per product, which this count does NOT include."""
    hq, hk = s.n_heads * s.head_dim, s.n_kv_heads * s.head_dim
    proj = (hq + 2 * hk) * s.d_model + s.d_model * hq + 3 * s.d_ffn * s.d_model
    attn = 2 * hq * (n * (n + 1) // 2)
    return 2 * (s.n_layers * (n * proj + attn) + s.vocab * s.d_model)


def mean_context(n_prompt, window, warm, steps, tokens_per_step):
    """Mean cache length over the timed speculative steps: the window is rewound to the prompt every `window` steps
    (counted from the first untimed step on) and grows by the committed tokens of a step."""
    pos = [(warm + i) % window for i in range(steps)]
    return n_prompt + tokens_per_step * (sum(pos) / max(1, len(pos)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--min-warmup-s", type=float, default=2.0,
                    help="after the --warmup steps, go on with untimed steps until this many seconds have passed since "
                         "the warm-up began: the first process on an idle GPU otherwise measures 2-3 %% below the steady "
                         "state that later runs on the same box show (0 = exactly --warmup steps)")
    ap.add_argument("--config", default="7b")
    ap.add_argument("--damp", type=float, default=1.0, help="skip-damping gamma (1 = verbatim config)")
    ap.add_argument("--K", type=int, default=None, help="speculation depth (default: the configuration's)")
    ap.add_argument("--sublayer-mask", default=None, metavar="A,F",
                    help="skip the fractions A of the attention and F of the FFN sub-layers (seeded, drawn "
                         "separately) instead of the configuration's whole layers, e.g. 0.5,0.35")
    ap.add_argument("--high-acceptance-damp", type=float, default=1e-5,
                    help="second, shorter speculative run on the same shape with this skip-damping gamma (an acceptance "
                         "rate in the paper's range), reported beside the verbatim workload's figure; 0 < gamma, "
                         "negative = skip that run")
    ap.add_argument("--fit", action="store_true",
                    help="measure the draft construction instead of the decode step: FIT layer scores (Eq. 11, Alg. 1 "
                         "Stage A) of the configuration over --fit-samples seeded sequences of --fit-tokens tokens; "
                         "prints its own JSON line")
    ap.add_argument("--fit-samples", type=int, default=4)
    ap.add_argument("--fit-tokens", type=int, default=512)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-run", action="store_true",
                    help="short run for `rocprofv3 --pmc`: prefill, a 1 GiB device copy (counter calibration), "
                         "two speculative steps, two plain decode steps; prints no benchmark line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (batch-1 decode step; no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    from synth.device import DeviceWeights
    import paper_2602_05499_amd as P

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    P.load_library()
    s = synth.CONFIGS[args.config]
    if args.fit:
        fit_bench(args, s, P, synth, DeviceWeights, np, torch)
        return
    if args.K is not None:
        s = s.with_(K=args.K)
    K = s.K
    mode = P.SD_GREEDY if s.mode == "greedy" else P.SD_SAMPLE
    if args.sublayer_mask:
        fa, ff = (float(x) for x in args.sublayer_mask.split(","))
        mask = synth.gen_sublayer_mask(s, fa, ff)
    else:
        mask = synth.gen_skip_mask(s)
    L_d = int((mask == 0).sum())
    n_attn_d, n_ffn_d = int(((mask & 1) == 0).sum()), int(((mask & 2) == 0).sum())
    torch.cuda.set_device(0)
    dw = DeviceWeights(s, damp_skipped=args.damp, skip_mask=mask)
    ses = P.Session(s, dw, mask, max_seq=s.max_seq, max_k=K, max_out=(args.steps + args.warmup + EXTRA_WARMUP_MAX + 2) * (K + 1) + 8)
    prompt = synth.gen_prompt(synth.SEED_PROMPT, s.n_prompt, s.vocab)
    n_uni = 1 + (2 * K + 1) * (args.steps + args.warmup + EXTRA_WARMUP_MAX + 1)
    uni = synth.gen_uniforms(synth.SEED_UNIFORMS, n_uni)
    # steps per generation window: rewind the cache length to the prompt's when the window is used up, so the
    # context stays within [n_prompt, n_prompt + n_gen) as in the configuration (KV already in HBM)
    window = max(1, (s.n_gen - 1) // (K + 1))

    if args.pmc_run:
        # steps at the mean context of the default run's timed steps (one committed token per step): the prompt is
        # simply that long here, so the counters and the bench line's algorithmic bytes speak of the same context
        ctx_pmc = int(round(mean_context(s.n_prompt, window, 0, window, 1.0)))
        prompt = synth.gen_prompt(synth.SEED_PROMPT, ctx_pmc, s.vocab)
        ses.prefill(prompt, mode, uni[0:1] if mode == P.SD_SAMPLE else None)
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB read + 1 GiB written
        b = torch.empty_like(a)
        b.copy_(a)
        for i in range(2):
            u = uni[1 + i * (2 * K + 1):1 + (i + 1) * (2 * K + 1)] if mode == P.SD_SAMPLE else None
            ses.draft(K, mode, None if u is None else u[:K]); ses.verify()
            ses.accept(mode, None if u is None else u[K:]); ses.rollback()
        for i in range(2):
            ses.decode(mode, uni[-1:] if mode == P.SD_SAMPLE else None)
        ses.sync()
        print(json.dumps({"pmc_run": True, "calibration_copy_bytes_each_way": a.numel() * 4, "context": ctx_pmc,
                          "algorithmic_bytes": {"verify": algorithmic_bytes(s, s.n_layers, s.n_layers, K + 1, ctx_pmc + K + 1),
                                                "draft_forward": algorithmic_bytes(s, n_attn_d, n_ffn_d, 1, ctx_pmc + 1),
                                                "plain_decode": algorithmic_bytes(s, s.n_layers, s.n_layers, 1, ctx_pmc + 1)},
                          "prompt_flops": prompt_flops(s, ctx_pmc)}))
        ses.close()
        return

    warm_run = {}   # untimed steps actually run per kind

    def run(kind, n_warm, n_steps):
        """kind: 'sd' or 'plain'.  Returns (seconds, committed tokens, per-phase ms lists).  Uses the session that
        `ses` names when it is called."""
        t0 = time.time()
        ses.prefill(prompt, mode, uni[0:1] if mode == P.SD_SAMPLE else None)
        ses.sync()
        t_prefill = time.time() - t0
        _, st0 = ses.read(0)
        first = int(st0["t_last"])
        cur = 1
        ev = []
        stream_ctx = torch.cuda.current_stream()

        def one_step(timed):
            nonlocal cur
            if kind == "sd":
                if mode == P.SD_SAMPLE:
                    u = uni[cur:cur + 2 * K + 1]; cur += 2 * K + 1
                    e = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if timed else None
                    if timed: e[0].record(stream_ctx)
                    ses.draft(K, mode, u[:K])
                    if timed: e[1].record(stream_ctx)
                    ses.verify()
                    if timed: e[2].record(stream_ctx)
                    ses.accept(mode, u[K:])
                    ses.rollback()
                    if timed: e[3].record(stream_ctx); ev.append(e)
                else:
                    e = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if timed else None
                    if timed: e[0].record(stream_ctx)
                    ses.draft(K, mode)
                    if timed: e[1].record(stream_ctx)
                    ses.verify()
                    if timed: e[2].record(stream_ctx)
                    ses.accept(mode)
                    ses.rollback()
                    if timed: e[3].record(stream_ctx); ev.append(e)
            else:
                u = None
                if mode == P.SD_SAMPLE:
                    u = uni[cur:cur + 1]; cur += 1
                ses.decode(mode, u)

        win = window if kind == "sd" else s.n_gen - 1
        done = 0

        def loop(n, timed):
            nonlocal done
            for _ in range(n):
                if done and done % win == 0:
                    ses.set_pending(s.n_prompt, first)
                one_step(timed)
                done += 1

        t_warm = time.perf_counter()
        loop(n_warm, False)
        ses.sync()
        n_extra = 0
        while time.perf_counter() - t_warm < args.min_warmup_s and n_extra < EXTRA_WARMUP_MAX:
            loop(5, False)
            ses.sync()
            n_extra += 5
        warm_run[kind] = n_warm + n_extra
        _, st1 = ses.read(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        loop(n_steps, kind == "sd")
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        _, st2 = ses.read(0)
        committed = int(st2["committed"] - st1["committed"])
        phases = None
        if ev:
            phases = dict(draft=[e[0].elapsed_time(e[1]) for e in ev], verify=[e[1].elapsed_time(e[2]) for e in ev],
                          accept=[e[2].elapsed_time(e[3]) for e in ev])
        stats = {k: int(st2[k] - st1[k]) for k in ("steps", "drafted", "accepted", "examined")}
        return dt, committed, phases, stats, t_prefill

    dt_sd, tok_sd, ph, st_sd, t_prefill = run("sd", args.warmup, args.steps)
    dt_pl, tok_pl, _, _, _ = run("plain", args.warmup, args.steps)
    sd_tps = tok_sd / dt_sd
    pl_tps = tok_pl / dt_pl

    # the prompt forward on its own: warm, then 5 calls, each waited for (sd_prefill copies the prompt in and enqueues)
    def time_prefill(path_mode):
        ses.set_prefill_mode(path_mode)
        ts = []
        for rep in range(7):
            ses.sync(); t0 = time.perf_counter()
            ses.prefill(prompt, mode, uni[0:1] if mode == P.SD_SAMPLE else None)
            ses.sync(); ts.append(time.perf_counter() - t0)
        ses.set_prefill_mode(-1)
        return float(np.median(ts[2:]))
    # what the memory system gives a plain device-to-device copy (context for the roofline fractions; 8 TB/s is the
    # published peak, not what any kernel reaches here)
    def copy_rate():
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)   # 1 GiB
        b = torch.empty_like(a)
        b.copy_(a); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            b.copy_(a)
        e1.record(); torch.cuda.synchronize()
        return 10 * 2 * a.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    copy_gbs = copy_rate()
    matrix_ok = s.dtype == "bf16"
    t_pf = time_prefill(1) if matrix_ok else None
    t_pf_chunks = time_prefill(0)
    high = None
    if args.high_acceptance_damp >= 0 and not args.sublayer_mask:
        # the same step on weights whose skipped layers contribute gamma times their output: acceptance in the range the
        # paper reports.  Same kernels, same bytes; only the number of committed tokens per step changes.
        ses_main = ses
        # A second set of weights next to the first: where the device cannot hold both and the tiled copy (the 70B shape:
        # 138 + 138 + 128 GB), the main context gives up its copy for the duration and the second context runs without
        # one (its decode forwards then read the O and down projections row-major, 1.5-2 % slower).
        torch.cuda.empty_cache()
        tiled_main = 0 if ses_main.tiled is None else ses_main.tiled.numel()
        room = torch.cuda.mem_get_info()[0] - (dw.nbytes() + ses_main.kv.numel() + ses_main.ws.numel()) - (2 << 30)
        lend = tiled_main > 0 and room < tiled_main
        if lend:
            ses_main.set_tiled_weights(False)
            torch.cuda.empty_cache()
        dw_h = DeviceWeights(s, damp_skipped=args.high_acceptance_damp, skip_mask=mask)
        ses = P.Session(s, dw_h, mask, max_seq=s.max_seq, max_k=K,
                        max_out=(args.steps + args.warmup + EXTRA_WARMUP_MAX + 2) * (K + 1) + 8)
        warm_main = dict(warm_run)
        dt_h, tok_h, _, st_h, _ = run("sd", args.warmup, args.steps)
        warm_run.update(warm_main)   # the record of the main runs is what the line reports
        tiled_h = ses.tiled is not None
        ses.close()
        del dw_h
        ses = ses_main
        if lend:
            torch.cuda.empty_cache()
            ses_main.set_tiled_weights(True)
        high = {"skip_damping": args.high_acceptance_damp,
                "acceptance_rate": round(st_h["accepted"] / max(1, st_h["drafted"]), 4),
                "tokens_per_step": round(tok_h / args.steps, 4), "sd_tokens_per_s": round(tok_h / dt_h, 3),
                "sd_over_plain": round(tok_h / dt_h / pl_tps, 4), "tiled_weights": tiled_h}
    draft_ms = float(np.mean(ph["draft"]))
    verify_ms = float(np.mean(ph["verify"]))
    accept_ms = float(np.mean(ph["accept"]))
    plain_ms = dt_pl / args.steps * 1e3
    # contexts the timed launches really ran at (the KV term of the algorithmic bytes): a speculative window is rewound
    # every `window` steps and advances by the committed tokens of a step; a verify launch reads the cache of the step's
    # start plus its own K + 1 rows, draft launch i that cache plus i + 1 rows (mean (K + 1) / 2)
    ctx_sd = mean_context(s.n_prompt, window, warm_run["sd"], args.steps, tok_sd / args.steps)
    ctx_pl = mean_context(s.n_prompt, s.n_gen - 1, warm_run["plain"], args.steps, 1.0)
    b_verify = algorithmic_bytes(s, s.n_layers, s.n_layers, K + 1, ctx_sd + K + 1)
    b_draft1 = algorithmic_bytes(s, n_attn_d, n_ffn_d, 1, ctx_sd + (K + 1) / 2.0)
    b_plain = algorithmic_bytes(s, s.n_layers, s.n_layers, 1, ctx_pl + 1)
    step_ms = dt_sd / args.steps * 1e3
    gbs_verify = b_verify / (verify_ms * 1e-3) / 1e9
    gbs_draft = K * b_draft1 / (draft_ms * 1e-3) / 1e9
    gbs_plain = b_plain / (plain_ms * 1e-3) / 1e9
    c = (draft_ms / K) / plain_ms
    vr = verify_ms / plain_ms

    def proj(alpha):
        e = (K + 1.0) if alpha >= 1.0 else (1.0 - alpha ** (K + 1)) / (1.0 - alpha)
        return e / ((draft_ms + verify_ms + accept_ms) / plain_ms)

    alpha_meas = st_sd["accepted"] / max(1, st_sd["drafted"])
    out = {
        "metric": "committed tokens/s SD vs plain decode, batch 1; draft/verify HBM GB/s",
        "value": round(sd_tps, 3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "warmup_steps_run": warm_run,
        "ms_per_step": round(dt_sd / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if s.dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.config}: {s.n_layers}L d{s.d_model} H{s.n_heads}/{s.n_kv_heads} F{s.d_ffn} "
                               f"V{s.vocab} {s.dtype}; draft skips " +
                               (f"{s.n_layers - n_attn_d} attention and {s.n_layers - n_ffn_d} FFN sub-layers"
                                if args.sublayer_mask else f"{s.n_layers - L_d} layers") + f" (seeded mask), K={K}, "
                               f"{s.mode}, batch 1, prompt {s.n_prompt}, window {s.n_gen}",
                   "skip_damping": args.damp},
        "sd_tokens_per_s": round(sd_tps, 3), "plain_tokens_per_s": round(pl_tps, 3),
        "sd_over_plain_measured": round(sd_tps / pl_tps, 4),
        "sd_at_high_acceptance": high,
        "acceptance_rate_measured": round(alpha_meas, 4),
        "tokens_per_step_measured": round(tok_sd / args.steps, 4),
        "draft_ms_per_step": round(draft_ms, 4), "verify_ms_per_step": round(verify_ms, 4),
        "accept_rollback_ms_per_step": round(accept_ms, 4), "plain_decode_ms_per_token": round(plain_ms, 4),
        "prefill_s": round(t_prefill, 3),
        "prefill": prefill_record(s, t_pf, t_pf_chunks, 0 if ses.tiled is None else ses.tiled.numel()),
        "context_mean": {"speculative_steps": round(ctx_sd, 1), "plain_decode": round(ctx_pl, 1)},
        "hbm_gbs": {"draft": round(gbs_draft, 1), "verify": round(gbs_verify, 1), "plain_decode": round(gbs_plain, 1),
                    "peak": HBM_PEAK_GBS, "device_copy_1gib_read_plus_write": round(copy_gbs, 1)},
        "cost_ratio_draft_over_plain": round(c, 4), "cost_ratio_verify_over_plain": round(vr, 4),
        "projected_speedup_vs_alpha": {str(a): round(proj(a), 3) for a in (0.0, 0.5, 0.8, 0.9, 0.95, 0.98, 1.0)},
        "paper_reported": {"speedup": "1.32x-1.5x (LLaMA-2-13B, alpha 0.95-0.98, hardware unstated)"},
        "roofline": {"bound": "hbm", "kernel": "verify forward ((K+1)-row full model)",
                     "achieved": round(gbs_verify, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs_verify / HBM_PEAK_GBS, 4), "traffic": measured_traffic(args.config),
                     "traffic_context": measured_traffic(args.config, "context"),
                     "mfma_util": measured_traffic(args.config, "verify_mfma_util"),
                     "dominant_by_time": "draft_forward" if draft_ms > verify_ms else "verify_forward",
                     "algorithmic_bytes_per_launch": b_verify, "avg_launch_ms": round(verify_ms, 4),
                     "draft_frac": round(gbs_draft / HBM_PEAK_GBS, 4),
                     # both forward kernels of the step, and the step as a whole (K draft launches + one verify launch;
                     # the accept and rollback kernels move no bytes to speak of)
                     "kernels": {
                         "draft_forward": {"launches_per_step": K, "avg_launch_ms": round(draft_ms / K, 4),
                                           "algorithmic_bytes_per_launch": b_draft1, "achieved": round(gbs_draft, 1),
                                           "frac": round(gbs_draft / HBM_PEAK_GBS, 4),
                                           "share_of_step": round(draft_ms / step_ms, 4),
                                           "traffic": measured_traffic(args.config, "draft")},
                         "verify_forward": {"launches_per_step": 1, "avg_launch_ms": round(verify_ms, 4),
                                            "algorithmic_bytes_per_launch": b_verify, "achieved": round(gbs_verify, 1),
                                            "frac": round(gbs_verify / HBM_PEAK_GBS, 4),
                                            "share_of_step": round(verify_ms / step_ms, 4),
                                            "traffic": measured_traffic(args.config, "verify")}},
                     "step_frac": round((K * b_draft1 + b_verify) / (step_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
    }
    ses.close()

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(s, dw, mask, K, mode)
    print(json.dumps(out))


def fit_flops(s, T):
    """Multiply-add flops (2 per MAC) of one calibration sample as the method defines them, counted once: the forward
    products with every layer matrix and the output head, the same products again for the gradient with respect to
    their inputs, causal attention forward and backward, and the gradient norms of the weight matrices taken as
    || dY^T X ||^2 through two T x T Gram matrices per matrix (T^2 (in + out) MACs; the inputs' Gram matrices are shared
    by the matrices that read the same input)."""
    hq, hk = s.n_heads * s.head_dim, s.n_kv_heads * s.head_dim
    proj = (hq + 2 * hk) * s.d_model + s.d_model * hq + 3 * s.d_ffn * s.d_model
    attn = 2 * hq * (T * (T + 1) // 2)
    gram = T * T * ((s.d_model + hq + s.d_model + s.d_ffn) + (hq + 2 * hk + s.d_model + 2 * s.d_ffn + s.d_model))
    return 2 * (s.n_layers * (2 * T * proj + 3 * attn + gram) + 2 * T * s.vocab * s.d_model)


def fit_bench(args, s, P, synth, DeviceWeights, np, torch):
    """FIT layer scores of the configuration on seeded calibration sequences: one untimed sample, then the timed call."""
    from paper_2602_05499_amd.session import fit_scores
    from paper_2602_05499_amd import binding as B
    torch.cuda.set_device(0)
    dw = DeviceWeights(s)
    T, N = args.fit_tokens, args.fit_samples
    samples = np.stack([synth.gen_prompt(synth.SEED_PROMPT + 100 + i, T, s.vocab) for i in range(N)])
    fit_scores(s, dw, samples[:1])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ta, tf, ls = fit_scores(s, dw, samples)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    fl = fit_flops(s, T)
    tfl = fl * N / dt / 1e12
    rc, mask = B.sd_fit_prune_mask(ta, tf, s.n_skip / s.n_layers)
    out = {"metric": "FIT layer scores (Eq. 11): calibration tokens/s", "value": round(N * T / dt, 1), "unit": "tokens/s",
           "n_gpus": 1, "steps": N, "warmup": 1, "ms_per_step": round(dt / N * 1e3, 3), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32 activations, bf16 weights", "data": "synthetic",
           "config": {"workload": f"{args.config}: {s.n_layers}L d{s.d_model} H{s.n_heads}/{s.n_kv_heads} F{s.d_ffn} V{s.vocab} "
                                  f"{s.dtype}; {N} seeded sequences of {T} tokens (stand-in for the paper's WikiText2 calibration set)"},
           "roofline": {"bound": "mfma", "kernel": "whole pass (dominant kernel: the matrix-core GEMM of the prompt path, plain epilogue)",
                        "achieved": round(tfl, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(tfl / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                        "algorithmic_flops_per_sample": fl},
           "losses": [round(float(x), 4) for x in ls],
           "t_attn": [float(f"{x:.4g}") for x in ta], "t_ffn": [float(f"{x:.4g}") for x in tf],
           "prune_set_at_config_ratio": [int(l) for l in np.nonzero(mask)[0]]}
    if not args.no_cpu_baseline:
        from oracle.fit import fit_scores as oracle_fit
        small = s.with_(n_layers=2)
        hw = DeviceWeights(small).to_host()
        tt = 192
        t0 = time.perf_counter()
        oracle_fit(small, hw, [synth.gen_prompt(1, tt, s.vocab)])
        dtc = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(tt / dtc * 2 / s.n_layers, 3), "unit": "tokens/s", "kind": "oracle",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "sample": f"two layers of the same widths, one sequence of {tt} tokens in {dtc:.1f} s, scaled by "
                                         f"2/{s.n_layers} to the full depth (the oracle forms every weight gradient in float64)"}
    print(json.dumps(out))


def prefill_record(s, t_matrix, t_chunks, tiled_bytes=0):
    """The prompt forward against the matrix cores' peak.  `achieved` counts the method's flops once (see
    prompt_flops); `executed_mfma_frac` counts the three bfloat16 passes per product that the kernels really run."""
    fl = prompt_flops(s, s.n_prompt)
    rec = {"tokens": s.n_prompt, "chunk_path_ms": round(t_chunks * 1e3, 3), "algorithmic_flops": fl}
    if t_matrix is not None:
        tf = fl / t_matrix / 1e12
        rec.update({"ms": round(t_matrix * 1e3, 3), "path": "matrix-matrix (sd_set_prefill_mode 1; the default for this length)",
                    "tiled_weights_bytes": int(tiled_bytes),   # sd_set_tiled_weights: the layer matrices once more in tile order
                    "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                 "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                                 "executed_mfma_frac": round(3 * tf / MFMA_BF16_PEAK_TFLOPS, 4)}})
    else:
        rec.update({"ms": round(t_chunks * 1e3, 3), "path": "16-row chunks through the streaming kernel (float32 storage)"})
    return rec


def measured_traffic(config, which="verify"):
    """From the committed rocprofv3 --pmc summary of this configuration: HBM bytes per verify (or draft) launch
    (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a copy of known size), the context
    those launches ran at ("context"), or the verify kernel's MFMA utilisation ("verify_mfma_util").  None when no
    summary covers `config` or the summary lacks the figure."""
    path = os.path.join(ROOT, "profiles", f"forward_kernels_{config}_pmc.txt")
    key = which + ":" if which in ("context", "verify_mfma_util") else which + "_traffic_bytes_per_launch:"
    try:
        for line in open(path):
            if line.startswith(key):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(s, dw, mask, K, mode):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload: a short prompt,
    then a few speculative steps and a few plain decode tokens with the full-size model."""
    import numpy as np
    import synth
    from oracle import OracleModel, SpecDecoder
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    hw = dw.to_host()
    n_prompt, n_steps, n_plain = 16, 2, 3
    orc = OracleModel(s, hw, max_seq=n_prompt + (n_steps + 1) * (K + 1) + n_plain + 2)
    prompt = synth.gen_prompt(synth.SEED_PROMPT, n_prompt, s.vocab)
    sd = SpecDecoder(orc, mask, K, "greedy" if mode == 0 else "sample")
    uni = synth.gen_uniforms(synth.SEED_UNIFORMS, 1 + (2 * K + 1) * (n_steps + 1))
    sd.prefill(prompt, float(uni[0]) if mode else None)
    t0 = time.perf_counter()
    cur = 1
    n_tok = 0
    for _ in range(n_steps):
        n_tok += len(sd.step(uni[cur:cur + 2 * K + 1] if mode else None)); cur += 2 * K + 1
    dt_sd = time.perf_counter() - t0
    t0 = time.perf_counter()
    P0, tok = sd.P, sd.t_last
    for i in range(n_plain):
        z = orc.forward([tok], P0 + i)[0]
        tok = int(np.argmax(z.astype(np.float32)))
    dt_pl = time.perf_counter() - t0
    return {"value": round(n_tok / dt_sd, 4), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "plain_tokens_per_s": round(n_plain / dt_pl, 4),
            "sample": f"full-size model, {n_prompt}-token prompt, {n_steps} speculative steps (K={K}) = {n_tok} "
                      f"committed tokens in {dt_sd:.1f} s, then {n_plain} plain decode tokens in {dt_pl:.1f} s"}


if __name__ == "__main__":
    main()
