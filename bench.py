#!/usr/bin/env python3
"""Benchmark of the CLaSp hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input: K draft steps with the current skip set,
one verify forward over the K+1 rows, greedy acceptance on the host, and one DP layer selection on the last accepted
token's stored states. Prints ONE JSON line:
  metric/value : draft tokens/s of the layer-skipped draft model (1 / mean clasp_draft_step time), inputs resident
  dp_select_ms : mean time of one clasp_dp_select call (one per verify step)
  roofline     : the dominant kernel (gate/up SwiGLU GEMM) against the 8 TB/s HBM peak, its duration measured with
                 HIP events around each of its launches in the timed region
  cpu_baseline : the fp64 CPU oracle timed on the host cores on the same shapes
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the dominant kernel from rocprofv3 PMC runs (FETCH_SIZE + WRITE_SIZE, each scaled by what the
# counter reads for a 1 GiB copy); see profiles/gate_up_gemm_llama3-8b-shape_hbm_traffic.md. The projection runs as two
# kernels (up to 8 rows: 236.0 + 1.84 MB, above: 236.8 + 1.84 MB); a step of the default workload launches them 128 : 15.
MEASURED_TRAFFIC = {"llama3-8b-shape": (128 * (236.0e6 + 1.84e6) + 15 * (236.8e6 + 1.84e6)) / 143}

WORKLOADS = {
    # benchmark configuration 2: the one the metric is quoted on
    "llama3-8b-shape/T512/M12/K4": dict(shape="llama3-8b-shape", T=512, M=12, K=4),
    # benchmark configuration 1: small case the oracle finishes in seconds
    "tiny-f32/T64/M3/K4": dict(shape="tiny-f32", T=64, M=3, K=4),
    # benchmark configurations 5 (closed loop shape), 3 (context sweep) and 4 (70B shape)
    "llama3-8b-shape/T4096/M12/K6": dict(shape="llama3-8b-shape", T=4096, M=12, K=6),
    "llama3-8b-shape/T2048/M12/K4": dict(shape="llama3-8b-shape", T=2048, M=12, K=4),
    "llama3-8b-shape/T8192/M12/K4": dict(shape="llama3-8b-shape", T=8192, M=12, K=4),
    "llama3-8b-shape/T2048/M8/K4": dict(shape="llama3-8b-shape", T=2048, M=8, K=4),
    "llama3-8b-shape/T2048/M16/K4": dict(shape="llama3-8b-shape", T=2048, M=16, K=4),
    "llama3-8b-shape/T8192/M8/K4": dict(shape="llama3-8b-shape", T=8192, M=8, K=4),
    "llama3-8b-shape/T8192/M16/K4": dict(shape="llama3-8b-shape", T=8192, M=16, K=4),
    "llama3-8b-shape/T32768/M12/K4": dict(shape="llama3-8b-shape", T=32768, M=12, K=4),
    "llama3-8b-shape/T32768/M8/K4": dict(shape="llama3-8b-shape", T=32768, M=8, K=4),
    "llama3-8b-shape/T32768/M16/K4": dict(shape="llama3-8b-shape", T=32768, M=16, K=4),
    "llama3-70b-shape/T1024/M32/K4": dict(shape="llama3-70b-shape", T=1024, M=32, K=4),
}


def build_engine(shape, seed, max_seq, max_rows, keep_host=False, resid_scale=1.0):
    """Generates the random-init model layer by layer on the GPU and packs it; optionally keeps host copies."""
    import torch
    import synth_inputs as si
    import paper_2505_24196_amd as clasp
    eng = clasp.Engine(shape, max_seq=max_seq, max_rows=max_rows)
    host = {"layers": []} if keep_host else None
    head = si.gen_head(shape, seed, "cuda")
    eng.set_head(head["embed"], head["lm_head"], head["final_norm"])
    if keep_host:
        host.update({k: si.to_numpy(v) for k, v in head.items()})
    del head
    for l in range(shape.n_layers):
        w = si.gen_layer(shape, seed, l, "cuda", resid_scale)
        eng.set_layer(l, w)
        if keep_host:
            host["layers"].append({k: si.to_numpy(v) for k, v in w.items()})
        del w
    torch.cuda.empty_cache()
    eng.create()
    return eng, host


def algorithmic_bytes(shape, T, M):
    """Bytes the method itself must move: weights of each evaluated layer once, the shared KV prefix once per layer."""
    eb = shape.elem_bytes()
    wl = shape.layer_weight_elems() * eb
    kv = 2 * shape.kv_dim * eb * T
    head = shape.vocab * shape.d_model * eb
    L = shape.n_layers
    return {"dp_select": (L - 1) * (wl + kv), "draft_step": (L - M) * (wl + kv) + head,
            "verify_forward": L * (wl + kv) + head, "gate_up_kernel": 2 * shape.d_model * shape.d_ffn * eb,
            "kv_share_per_layer": kv / (wl + kv)}


def timed_calls(eng, shape, T, M, K, n=10):
    """Mean times of clasp_verify_forward (K+1 rows), clasp_dp_select and clasp_draft_step on a synthetic prefix of T
    tokens (drawn per layer on the device and installed with clasp_kv_load), each with its algorithmic bytes and the
    fraction of the 8 TB/s peak. Reuses a loaded engine: only the cache contents change."""
    import torch
    import synth_inputs as si
    for l in range(shape.n_layers):
        Kp, Vp = si.gen_kv(shape, 1000 + l, 1, T, "cuda")
        eng.clasp_kv_load(l, Kp[0], Vp[0])
    del Kp, Vp
    tok = si.gen_tokens(2, K + 1, shape.vocab, stream=9).cuda()
    ver = eng.clasp_verify_forward(tok, T, want_hidden=True)
    states = ver["hidden"][:, 1, :].contiguous()
    dp = eng.clasp_dp_select(states, T + 1, M)
    mask = dp["mask"].cpu().tolist()
    nxt = torch.zeros(1, dtype=torch.int32, device="cuda")
    eng.clasp_draft_step(mask, tok[:1], T + K + 1, nxt)
    torch.cuda.synchronize()
    e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    e[0].record()
    for _ in range(n):
        eng.clasp_verify_forward(tok, T, want_hidden=True)
    e[1].record()
    for _ in range(n):
        eng.clasp_dp_select(states, T + 1, M, out=dp)
    e[2].record()
    for _ in range(n):
        eng.clasp_draft_step(mask, tok[:1], T + K + 1, nxt)
    e[3].record()
    torch.cuda.synchronize()
    ms = {"verify_forward": e[0].elapsed_time(e[1]) / n, "dp_select": e[1].elapsed_time(e[2]) / n,
          "draft_step": e[2].elapsed_time(e[3]) / n}
    ab = algorithmic_bytes(shape, T, M)
    return {"context_tokens": T, "skip_budget_M": M, "calls_timed": n,
            "dp_select_ms": round(ms["dp_select"], 4), "draft_step_ms": round(ms["draft_step"], 4),
            "draft_tokens_per_s": round(1e3 / ms["draft_step"], 1), "verify_forward_ms": round(ms["verify_forward"], 4),
            "algorithmic_GB": {k: round(ab[k] / 1e9, 3) for k in ms},
            "hbm_frac_of_8TBs": {k: round(ab[k] / (v * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) for k, v in ms.items()},
            "kv_share_of_layer_bytes": round(ab["kv_share_per_layer"], 4)}


def closed_loop_run(eng, shape, T, M, K, n_gen):
    """Benchmark configuration 5 on a loaded engine: plain greedy decoding and the Draft -> Verify -> Layer-Optimisation
    loop over the same T-token prompt, n_gen tokens each (prompt pass included in both times), compared token for
    token. Between the two, the row-count check: plain decoding's own sequence is fed back K+1 rows at a time through
    clasp_verify_forward (the launch shape of a verify pass) and every row's greedy token is compared with what the
    one-row launches of plain decoding produced at that position - the lossless claim holds on the device exactly as
    far as a row's result does not depend on how many rows share its launch."""
    import torch
    import synth_inputs as si
    from paper_2505_24196_amd import decode
    prompt = [int(t) for t in si.gen_tokens(2, T, shape.vocab)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plain, margins = decode.greedy_generate(eng, prompt, n_gen)
    torch.cuda.synchronize()
    t_plain = time.perf_counter() - t0
    # plain[i] sits at position T + i; a verify pass over rows plain[s .. s+K] at positions T+s.. predicts plain[s+1 ..]
    seq = torch.as_tensor(plain, dtype=torch.int32, device=eng.device)
    differs = []
    compared = 0
    for s0 in range(0, n_gen - 1, K + 1):
        rows = seq[s0:min(s0 + K + 1, n_gen - 1)]
        out = eng.clasp_verify_forward(rows, T + s0, want_margin=True)
        got = out["argmax"].cpu().tolist()
        for r, g in enumerate(got):
            compared += 1
            if g != plain[s0 + r + 1]:
                differs.append({"position": T + s0 + r, "plain_margin": round(margins[s0 + r + 1], 6),
                                "verify_margin": round(float(out["margin"][r]), 6)})
    t0 = time.perf_counter()
    spec = decode.clasp_generate(eng, prompt, n_gen, M, K)
    torch.cuda.synchronize()
    t_spec = time.perf_counter() - t0
    first_diff = next((i for i, (a, b) in enumerate(zip(plain, spec["tokens"])) if a != b), None)
    acc = [r["accepted"] for r in spec["rounds"]]
    return {"workload": f"{shape.name}/T{T}/M{M}/K{K}", "generated": n_gen, "includes_prompt_pass": True,
            "plain_greedy_tokens_per_s": round(n_gen / t_plain, 2), "clasp_tokens_per_s": round(n_gen / t_spec, 2),
            "speedup": round(t_plain / t_spec, 3), "rounds": len(acc),
            "mean_tokens_per_round": round(n_gen / max(1, len(acc)), 3),
            "tokens_equal": first_diff is None, "first_difference_at": first_diff,
            "plain_margin_at_difference": None if first_diff is None else margins[first_diff],
            "smallest_plain_margin": round(min(margins), 6),
            "row_count_check": {"rows_per_launch": K + 1, "positions_compared": compared,
                                "greedy_token_differs": len(differs), "where": differs[:8]},
            "note": "random-init weights: draft and full model rarely agree, so the loop is slower than plain decoding; "
                    "the figure that carries over to trained weights is the per-call cost"}


def cpu_baseline(shape, host_model, T, M, budget_s=30.0):
    """Times the oracle (as it stands) on the host cores: one DP layer selection and one draft step on the same model,
    with a seeded synthetic KV prefix of T tokens standing in for the prefill the oracle cannot afford."""
    import numpy as np
    import synth_inputs as si
    from oracle import clasp_oracle as oc
    om = oc.OracleModel(shape, host_model)
    cache = oc.KVCache(shape, T + 8)
    K, V = si.gen_kv(shape, 3, shape.n_layers, T)
    cache.load(K.numpy().astype(np.float64), V.numpy().astype(np.float64))
    del K, V
    tok = int(si.gen_tokens(2, 1, shape.vocab, stream=7)[0])
    t0 = time.time()
    states, _ = om.token(tok, T, cache, want_states=True)
    t_verify_row = time.time() - t0
    # bound the sample: the DP costs about sum_i min(i-1, M) row-layers, one verify row costs L of them
    L = shape.n_layers
    row_layers = sum(min(i - 1, M) for i in range(1, L + 1))
    est = t_verify_row / L * row_layers
    M_s = M
    while M_s > 1 and est > budget_s:
        M_s -= 1
        est = t_verify_row / L * sum(min(i - 1, M_s) for i in range(1, L + 1))
    t0 = time.time()
    res = om.dp(states, T, cache, M_s)
    t_dp = time.time() - t0
    scale = row_layers / max(1, sum(min(i - 1, M_s) for i in range(1, L + 1)))
    t0 = time.time()
    om.token(tok, T, cache, skip=res["mask"] if M_s == M else None)
    t_draft = time.time() - t0
    if M_s != M:
        t_draft *= (L - M) / L
    return {"value": round(1.0 / t_draft, 3), "unit": "draft tokens/s", "cores": oc.num_threads(), "kind": "oracle",
            "dp_select_ms": round(t_dp * scale * 1e3, 1), "verify_row_ms": round(t_verify_row * 1e3, 1),
            "sample": f"one oracle DP with M={M_s} (scaled x{scale:.2f} to M={M}), one draft step and one verify row "
                      f"(the full model on one token; a verify pass is K+1 of them) at T={T} on synthetic KV, {shape.name}"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3-8b-shape/T512/M12/K4", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timer", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="default workload only: leave out the context sweep (T = 2048 / 8192 / 32768) and the 512-token "
                         "closed loop of benchmark configuration 5 that otherwise follow the timed steps on the same engine")
    ap.add_argument("--closed-loop", type=int, default=0, metavar="N_TOKENS",
                    help="instead of the step benchmark: generate N_TOKENS with the full draft/verify/optimise loop and "
                         "with plain greedy decoding on the chosen workload, compare the tokens, report tokens/s of both")
    ap.add_argument("--resid-scale", type=float, default=1.0,
                    help="closed loop only: std multiplier of wo / w_down (0.05 = slow-drift variant whose drafts get "
                         "accepted; 1.0 = the plain N(0, 0.02) init of the benchmark configurations)")
    ap.add_argument("--dp-interval", type=int, default=1,
                    help="closed loop only: re-optimise the skip set every this many verify steps (Sec. 3.7)")
    ap.add_argument("--det-threshold", type=float, default=None,
                    help="closed loop only: draft-exiting threshold on the draft token's top-1 probability (Sec. 5.3.3)")
    ap.add_argument("--temperature", type=float, default=None,
                    help="closed loop only: stochastic decoding at this temperature (speculative sampling with seeded "
                         "uniform numbers) instead of greedy decoding; reports rounds and acceptance, no token comparison")
    ap.add_argument("--markov-study", action="store_true",
                    help="only run the comparison of the paper's Sec. 3.5 on the workload's model: first and last 10/32 "
                         "of the layers fixed, skip sets of the layers between chosen by brute force, at random and by "
                         "the dynamic program; cosine of the resulting last hidden state with the full model's")
    ap.add_argument("--prefill", type=int, default=0, metavar="N_TOKENS",
                    help="only time the prompt pass (clasp_prefill) over N_TOKENS synthetic tokens of the workload's "
                         "model; prints its own JSON line (tokens/s, algorithmic TFLOP/s against the bf16 MFMA peak)")
    ap.add_argument("--prefill-chunk", type=int, default=4096, help="rows per pass of --prefill (multiple of 128)")
    ap.add_argument("--call", choices=["dp_select", "draft_step", "verify_forward"], default=None,
                    help="only issue this one call --steps times on the workload's model over a synthetic prefix of the "
                         "workload's length (after one warm-up round of all three calls): what a rocprofv3 run of a single "
                         "call's kernels is taken from; prints the call's mean time")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="only run plain device copies of a known size (1 GiB read + 1 GiB written per copy), to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    import synth_inputs as si
    import paper_2505_24196_amd as clasp
    from paper_2505_24196_amd import decode

    if args.pmc_calibration:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda")  # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "5 device copies, each reads 1 GiB and writes 1 GiB (1048576 KiB)"}))
        return

    wl = WORKLOADS[args.workload]
    shape = si.SHAPES[wl["shape"]]
    T, M, K = wl["T"], wl["M"], wl["K"]
    if args.call:
        eng, _ = build_engine(shape, 1, ((T + 64 + 31) // 32) * 32, 32 if M > 16 else 16)
        print("model loaded", file=sys.stderr, flush=True)
        for l in range(shape.n_layers):
            Kp, Vp = si.gen_kv(shape, 1000 + l, 1, T, "cuda")
            eng.clasp_kv_load(l, Kp[0], Vp[0])
        tok = si.gen_tokens(2, K + 1, shape.vocab, stream=9).cuda()
        ver = eng.clasp_verify_forward(tok, T, want_hidden=True)
        states = ver["hidden"][:, 1, :].contiguous()
        dp = eng.clasp_dp_select(states, T + 1, M)
        mask = dp["mask"].cpu().tolist()
        nxt = torch.zeros(1, dtype=torch.int32, device="cuda")
        eng.clasp_draft_step(mask, tok[:1], T + K + 1, nxt)
        torch.cuda.synchronize()
        print("prefix loaded, warm-up round done", file=sys.stderr, flush=True)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = max(1, args.steps)
        e0.record()
        for _ in range(n):
            if args.call == "dp_select":
                eng.clasp_dp_select(states, T + 1, M, out=dp)
            elif args.call == "draft_step":
                eng.clasp_draft_step(mask, tok[:1], T + K + 1, nxt)
            else:
                eng.clasp_verify_forward(tok, T, want_hidden=True)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / n
        ab = algorithmic_bytes(shape, T, M)[args.call]
        print(json.dumps({"call": args.call, "workload": args.workload, "calls": n, "warmup_calls_of_each_kind": 1,
                          "ms_per_call": round(ms, 4), "algorithmic_GB": round(ab / 1e9, 3),
                          "hbm_frac_of_8TBs": round(ab / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}))
        return
    if args.markov_study:
        eng, _ = build_engine(shape, 1, ((T + 64 + 31) // 32) * 32, 16, resid_scale=args.resid_scale)
        Kp, Vp = si.gen_kv(shape, 3, 1, T, "cuda")
        for l in range(shape.n_layers):
            eng.clasp_kv_load(l, Kp[0], Vp[0])
        tok = si.gen_tokens(2, 1, shape.vocab, stream=9).cuda()
        states = eng.clasp_verify_forward(tok, T, want_hidden=True)["hidden"][:, 0].contiguous()
        lo = 10 * shape.n_layers // 32
        hi = shape.n_layers - lo
        budgets = [m for m in (2, 4, 6, 8, 10) if m < hi - lo]
        t0 = time.perf_counter()
        rows = decode.markov_study(eng, states, tok, T, lo, hi, budgets)
        torch.cuda.synchronize()
        print(json.dumps({"markov_study": args.workload, "resid_scale": args.resid_scale, "window": [lo, hi],
                          "seconds": round(time.perf_counter() - t0, 2), "rows": rows}))
        return
    if args.prefill:
        n = args.prefill
        eng, _ = build_engine(shape, 1, ((n + 31) // 32) * 32, 16)
        toks = si.gen_tokens(2, n, shape.vocab).cuda()
        for _ in range(max(1, args.warmup)):
            eng.clasp_prefill(toks, 0, args.prefill_chunk)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        steps = max(1, args.steps)
        e0.record()
        for _ in range(steps):
            eng.clasp_prefill(toks, 0, args.prefill_chunk)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        # algorithmic flops: every projection of layers 0..L-2 plus the last layer's q/k/v (nothing after it feeds the
        # cache), 2 flop per weight and row; causal attention 4 * q_dim flop per (query, visible key) pair
        L, d, F = shape.n_layers, shape.d_model, shape.d_ffn
        qd, kvd = shape.n_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
        p_qkv = d * (qd + 2 * kvd)
        p_layer = p_qkv + qd * d + 3 * d * F
        flops = 2.0 * n * ((L - 1) * p_layer + p_qkv) + (L - 1) * 4.0 * qd * n * (n + 1) / 2
        tf = flops / ms / 1e9
        # passes of 640 rows or more run on fp16 MFMAs (one fp16 operand per activation, weights converted per layer)
        f16_pass = min(n, args.prefill_chunk) >= 640
        note = ("algorithmic flops; projections on fp16 MFMAs (fp32 accumulation), attention on bf16" if f16_pass else
                "algorithmic flops; activations enter as bf16 hi + lo, so the matrix cores execute twice the GEMM flops "
                "counted here")
        print(json.dumps({"metric": "prefill_tokens_per_s", "value": round(n / ms * 1e3, 1), "unit": "tokens/s", "n_gpus": 1,
                          "steps": steps, "warmup": max(1, args.warmup), "ms_per_step": round(ms, 3),
                          "higher_is_better": True, "dtype": "f16" if f16_pass else "bf16", "data": "synthetic",
                          "config": {"workload": f"{shape.name}/prefill{n}/chunk{args.prefill_chunk}"},
                          "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": 2500.0, "unit": "TFLOP/s",
                                       "frac": round(tf / 2500.0, 4), "traffic": None, "note": note}}))
        return
    if args.closed_loop:
        n_gen = args.closed_loop
        max_seq = ((T + n_gen + K + 2 + 31) // 32) * 32
        eng, _ = build_engine(shape, 1, max_seq, 32 if M > 16 else 16, resid_scale=args.resid_scale)
        prompt = [int(t) for t in si.gen_tokens(2, T, shape.vocab)]
        torch.cuda.synchronize()
        if args.temperature is not None:
            un = {"first": si.gen_uniform(5, 1, 10).cuda(), "draft": si.gen_uniform(5, n_gen * K, 11).cuda(),
                  "accept": si.gen_uniform(5, n_gen * K, 12).cuda(), "final": si.gen_uniform(5, n_gen, 13).cuda()}
            t0 = time.perf_counter()
            spec = decode.clasp_sample_generate(eng, prompt, n_gen, M, K, un, args.temperature)
            torch.cuda.synchronize()
            t_spec = time.perf_counter() - t0
            acc = [r["accepted"] for r in spec["rounds"]]
            print(json.dumps({"closed_loop": args.workload, "temperature": args.temperature, "resid_scale": args.resid_scale,
                              "generated": n_gen, "includes_prefill": True, "clasp_tokens_per_s": round(n_gen / t_spec, 2),
                              "rounds": len(acc), "mean_accepted_drafts": round(sum(acc) / max(1, len(acc)), 3),
                              "skip_set_jaccard_by_round_gap": [round(x, 3) for x in decode.skip_set_jaccard(
                                  [r["mask"] for r in spec["rounds"]], 8)]}))
            return
        t0 = time.perf_counter()
        plain, margins = decode.greedy_generate(eng, prompt, n_gen)
        torch.cuda.synchronize()
        t_plain = time.perf_counter() - t0
        t0 = time.perf_counter()
        spec = decode.clasp_generate(eng, prompt, n_gen, M, K, dp_interval=args.dp_interval,
                                     det_threshold=args.det_threshold)
        torch.cuda.synchronize()
        t_spec = time.perf_counter() - t0
        first_diff = next((i for i, (a, b) in enumerate(zip(plain, spec["tokens"])) if a != b), None)
        acc = [r["accepted"] for r in spec["rounds"]]
        print(json.dumps({"closed_loop": args.workload, "resid_scale": args.resid_scale, "generated": n_gen, "includes_prefill": True,
                          "plain_greedy_tokens_per_s": round(n_gen / t_plain, 2),
                          "clasp_tokens_per_s": round(n_gen / t_spec, 2), "speedup": round(t_plain / t_spec, 3),
                          "rounds": len(acc), "mean_tokens_per_round": round(n_gen / max(1, len(acc)), 3),
                          "dp_interval": args.dp_interval, "det_threshold": args.det_threshold,
                          "skip_set_jaccard_by_round_gap": [round(x, 3) for x in decode.skip_set_jaccard(
                              [r["mask"] for r in spec["rounds"]][::args.dp_interval], 8)],
                          "tokens_equal": first_diff is None, "first_difference_at": first_diff,
                          "plain_margin_at_difference": None if first_diff is None else margins[first_diff]}))
        return
    total_steps = args.steps + args.warmup
    max_seq = ((T + (K + 1) * (total_steps + 2) + 31) // 32) * 32
    extras = (not args.no_extras) and args.workload == "llama3-8b-shape/T512/M12/K4"
    if extras:
        max_seq = max(max_seq, 32768 + 64)
    want_cpu = not args.no_cpu_baseline
    eng, host = build_engine(shape, 1, max_seq, 32 if M > 16 else 16, keep_host=want_cpu)
    dev = eng.device

    prompt = [int(t) for t in si.gen_tokens(2, T, shape.vocab)]
    states, nxt, _ = decode.prefill(eng, prompt)
    pos = T
    dp_out = eng.clasp_dp_select(states, pos - 1, M)
    mask = dp_out["mask"].cpu().tolist()
    tok = torch.empty(K + 1, dtype=torch.int32, device=dev)
    tok[0:1].copy_(nxt)
    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
    t_draft = t_verify = t_dp = 0.0
    accepted = 0
    pairs = []
    kt_ms, kt_n = 0.0, 0
    for step in range(total_steps):
        timed = step >= args.warmup
        if step == args.warmup:
            torch.cuda.synchronize()
            if not args.no_kernel_timer:
                eng.kernel_timer_begin("gate_up", every=8)  # sampled: each event pair costs the stream ~3 us
            t_start = time.perf_counter()
        e = [ev() for _ in range(4)]
        e[0].record()
        for k in range(K):
            eng.clasp_draft_step(mask, tok[k:k + 1], pos + k, tok[k + 1:k + 2])
        e[1].record()
        ver = eng.clasp_verify_forward(tok, pos, want_hidden=True)
        e[2].record()
        rows = tok.cpu().tolist()
        v = ver["argmax"].cpu().tolist()
        a = 0
        while a < K and rows[a + 1] == v[a]:
            a += 1
        e2 = ev()
        e2.record()
        eng.clasp_dp_select(ver["hidden"][:, a, :], pos + a, M, out=dp_out)
        e[3].record()
        mask = dp_out["mask"].cpu().tolist()
        tok[0:1].copy_(ver["argmax"][a:a + 1])
        pos += a + 1
        if timed:
            accepted += a
            pairs.append((e[0], e[1], e[2], e2, e[3]))
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_start
    if not args.no_kernel_timer:
        kt_ms, kt_n = eng.kernel_timer_end()
    for p in pairs:
        t_draft += p[0].elapsed_time(p[1])
        t_verify += p[1].elapsed_time(p[2])
        t_dp += p[3].elapsed_time(p[4])
    n = args.steps
    draft_ms = t_draft / (n * K)
    dp_ms = t_dp / n
    verify_ms = t_verify / n
    ab = algorithmic_bytes(shape, T, M)
    frac = lambda b, ms: round(b / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)  # noqa: E731
    out = {
        "metric": "DP-select ms/verify step + draft tokens/s (8B-shape, 1 GPU); % HBM roofline",
        "value": round(1e3 / draft_ms, 2), "unit": "draft tokens/s", "n_gpus": 1, "steps": n, "warmup": args.warmup,
        "ms_per_step": round(t_total * 1e3 / n, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "context_tokens": T, "skip_budget_M": M, "draft_len_K": K,
                   "layers": shape.n_layers, "d_model": shape.d_model, "weights": "random-init N(0,0.02), seed 1"},
        "dp_select_ms": round(dp_ms, 4), "draft_step_ms": round(draft_ms, 4), "verify_forward_ms": round(verify_ms, 4),
        "mean_accepted": round(accepted / n, 3), "tokens_per_s_closed_loop": round((accepted + n) / t_total, 2),
        "hbm_frac_of_8TBs": {"dp_select": frac(ab["dp_select"], dp_ms), "draft_step": frac(ab["draft_step"], draft_ms),
                             "verify_forward": frac(ab["verify_forward"], verify_ms)},
        "kv_share_of_layer_bytes": round(ab["kv_share_per_layer"], 4),
    }
    # achievable ceiling next to the nominal 8 TB/s: a plain device copy (1 GiB read + 1 GiB written per copy), untimed region
    src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(10):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2 * src.numel() * 2 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst
    if shape.dtype == "bf16":  # the prompt pass over a prompt of the workload's length (overwrites the synthetic prefix: last)
        ptoks = si.gen_tokens(2, T, shape.vocab).cuda()
        eng.clasp_prefill(ptoks, 0, min(4096, (T + 127) // 128 * 128))
        torch.cuda.synchronize()
        c0.record()
        for _ in range(3):
            eng.clasp_prefill(ptoks, 0, min(4096, (T + 127) // 128 * 128))
        c1.record()
        torch.cuda.synchronize()
        out["prompt_pass_ms"] = round(c0.elapsed_time(c1) / 3, 3)
    out["device_copy_GBs"] = round(copy_gbs, 1)
    out["frac_of_device_copy"] = {k: round(v * 8000.0 / copy_gbs, 4) for k, v in out["hbm_frac_of_8TBs"].items()}
    if kt_n:
        avg_ms = kt_ms / kt_n
        ach = ab["gate_up_kernel"] / (avg_ms * 1e-3) / 1e9
        out["roofline"] = {"bound": "hbm", "kernel": "gate|up projection + SwiGLU (gemv_persistent_bf16_kernel for <= 8 rows, gemm_bf16_resident_kernel above)" if shape.dtype == "bf16"
                           else "gemm_f32_kernel<SwiGLU> (gate/up projection)",
                           "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC.get(shape.name),
                           "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised under profiles/, "
                                             "not measured in this run",
                           "launches": kt_n,
                           "avg_us": round(avg_ms * 1e3, 2), "bytes_per_launch": ab["gate_up_kernel"]}
    if extras:  # benchmark configurations 3 (context sweep) and 5 (closed loop) on the same engine
        out["context_sweep"] = [timed_calls(eng, shape, Ts, M, K) for Ts in (2048, 8192, 32768)]
        out["closed_loop"] = closed_loop_run(eng, shape, 4096, 12, 6, 512)
    eng.close()
    del eng
    torch.cuda.empty_cache()
    if want_cpu:
        out["cpu_baseline"] = cpu_baseline(shape, host, T, M)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
