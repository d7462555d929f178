#!/usr/bin/env python3
"""Benchmark of the SDLM block-decode step on one MI355X.

A "step" is one pass of the whole hot path over the batch: row assembly, embedding, L decoder layers (RMSNorm,
QKV GEMM, RoPE + K/V placement, block-masked attention, O projection, gate/up GEMM + SwiGLU, down projection),
final norm, LM head with fused online softmax / arg-max, prefix acceptance, and the commit that publishes the
accepted tokens.  Inputs (weights, prompts) are synthetic and already resident in HBM when the clock starts.

Prints ONE JSON line: metric = accepted tokens/s over the timed steps, plus block-step latency, the roofline
object of the dominant kernel (HIP-event timed inside the timed region) and the CPU oracle baseline.
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
PEAK_BF16_TFLOPS = 2500.0    # dense MFMA bf16


MAIN_PHASES = ("attn", "attn_merge", "qkv", "oproj", "gateup", "down", "lmhead")


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload, if there is one
    (lines "traffic_bytes_per_launch <workload> <kernel> <bytes>" in profiles/*.txt)."""
    import glob
    for f in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(f):
            t = line.split()
            if len(t) == 4 and t[0] == "traffic_bytes_per_launch" and t[1] == workload and t[2] == kernel:
                return float(t[3])
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="C4", help="C1..C5 (default: the 7B-shaped workload the target is quoted on)")
    ap.add_argument("--tau", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true", help="also time the other thresholds of the workload's tau sweep")
    ap.add_argument("--phases", default="gateup",
                    help="phases bracketed by HIP events inside the timed region: phase names separated by commas (default: the dominant kernel), "
                         "main (all six big kernels, ~6%% slower steps) or none; the per-kernel table of the other phases comes "
                         "from up to 32 extra untimed steps")
    ap.add_argument("--profile-every", type=int, default=9,
                    help="inside the timed region only every n-th launch of a bracketed phase carries its two event records "
                         "(an event record between two kernels keeps them from running back to back); 9 is coprime to the "
                         "layer counts, so the samples rotate through the layers")
    ap.add_argument("--conf-fn", type=int, default=0, choices=(0, 1), help="0: softmax probability of the arg-max token; 1: entropy-normalised confidence")
    ap.add_argument("--accept-rule", type=int, default=0, choices=(0, 1), help="0: cumulative product >= tau (the paper's rule); 1: every leading confidence >= tau")
    ap.add_argument("--block-causal", action="store_true", help="the causal-in-block ablation instead of mutual attention inside the block")
    ap.add_argument("--force-accept", type=int, default=0,
                    help="commit this many of the step's tokens for every sequence instead of gamma (random weights accept about "
                         "1.05 tokens/step; this shows the step at a trained model's acceptance, e.g. 2). The reported rate "
                         "is then tokens committed/s, labelled as forced")
    ap.add_argument("--prefill-rows", type=int, default=0, help="rows per prefill pass (0: library default)")
    ap.add_argument("--verify", type=int, default=None, choices=(0, 1),
                    help="self-speculative decoding: every step is followed by the verification pass and commits gamma_verify "
                         "tokens (rule 0: agreeing prefix, 1: largest agreeing index); no per-kernel table in this mode")
    ap.add_argument("--graph", action="store_true",
                    help="replay the decode step as a HIP graph (library on a side stream); steps run eagerly while any phase "
                         "carries events, so combine with --phases none")
    ap.add_argument("--profile-all", action="store_true", help="bracket every phase with events (adds overhead)")
    return ap.parse_args()


def build_model(ctx, m, seed, keep_host_layers=None):
    """Generate weights on the GPU layer by layer and hand them to the library; optionally keep host copies."""
    import torch
    from paper_2509_24007_amd import inputs as syn
    g = syn.make_globals(m, seed, device="cuda")
    ctx.init_weights(g, None)
    host_g = {k: v.cpu() for k, v in g.items()} if keep_host_layers is not None else None
    torch.cuda.synchronize()
    del g
    host_layers = []
    for l in range(m.n_layers):
        L = syn.make_layer(m, seed, l, device="cuda")
        ctx.init_weights(None, {l: L})
        if keep_host_layers is not None and l < keep_host_layers:
            host_layers.append({k: (v.cpu() if v is not None else None) for k, v in L.items()})
        torch.cuda.synchronize()
        del L
    torch.cuda.empty_cache()
    return host_g, host_layers


def algorithmic_bytes(m, esz, lens_sum, R):
    """Bytes one step must move: every weight once, every cached K/V once, plus the small activations."""
    d, h, F, V = m.head_dim, m.hidden, m.ffn, m.vocab
    nq, nk = m.n_q_heads * d, m.n_kv_heads * d
    per_layer = (nq + 2 * nk) * h + h * nq + 3 * F * h
    weights = (per_layer * m.n_layers + V * h) * esz
    kv = lens_sum * 2 * nk * esz * m.n_layers
    return weights, kv


def run_tau(ctx, m, r, prompts, tau_idx, steps, warmup, prof_phases, table_steps=0, verify=None, force=0, every=1):
    """Warm-up, then the timed region (only `prof_phases` carry events: every bracketed phase costs two event records
    per launch), then `table_steps` untimed extra steps with every main phase bracketed for the per-kernel table."""
    import torch
    B, D = len(prompts), r.block_D
    torch.cuda.synchronize()
    tp = time.perf_counter()
    ctx.prefill(prompts)
    torch.cuda.synchronize()
    run_tau.prefill_s = time.perf_counter() - tp
    ids = torch.zeros(warmup + steps + table_steps, B, D, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(warmup + steps + table_steps, B, dtype=torch.int32, device="cuda")
    forced = torch.full((B,), force, dtype=torch.int32, device="cuda") if force else None
    torch.cuda.synchronize()

    def one(t):
        ctx.decode_step(ids[t], cnt[t])
        if verify is not None:
            ctx.verify_step(verify, None, cnt[t])      # the committed count becomes gamma_verify
        if forced is not None:
            ctx.kv_commit(ids[t], forced)
        else:
            ctx.kv_commit()
    for t in range(warmup):
        one(t)
    torch.cuda.synchronize()
    ctx.profile(prof_phases, every)
    # one event per step on the library's stream: the spread of the step's device time (median, p10, p90)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(ctx.stream)
    for t in range(warmup, warmup + steps):
        one(t)
        marks[t - warmup + 1].record(ctx.stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run_tau.step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    phases = ctx.profile_read()
    table = {}
    if table_steps:
        ctx.profile(MAIN_PHASES)
        for t in range(warmup + steps, warmup + steps + table_steps):
            one(t)
        torch.cuda.synchronize()
        table = ctx.profile_read()
    ctx.profile(None)
    n, c = ctx.get_lengths()
    return t1 - t0, cnt.cpu(), phases, n, table


def copy_ceiling(nbytes=1 << 30, reps=8):
    """A plain device-to-device copy (torch's copy kernel), the streaming rate this card reaches in practice: bytes read
    plus bytes written over the mean duration of `reps` copies."""
    import torch
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del src, dst
    torch.cuda.empty_cache()
    return {"GBs": 2 * nbytes / (ms * 1e-3) / 1e9, "copy_bytes": nbytes, "reps": reps,
            "kind": "device-to-device copy of one buffer, read + written bytes over the mean copy time"}


def weight_params(m):
    """Weight elements every row of a step is multiplied with: the projections of all layers and the LM head."""
    nq, nk = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    return m.n_layers * (m.hidden * (nq + 2 * nk) + nq * m.hidden + 3 * m.hidden * m.ffn) + m.vocab * m.hidden


def cpu_baseline(m, host_g, host_layers, prompt, D, tau, budget_s=12.0, max_steps=64, prompt_tokens=8, ctx_tokens=0.0):
    """The oracle as it stands, timed on a bounded sample: decode steps of one sequence until about budget_s seconds."""
    from oracle import oracle as orc
    om = orc.model_from_inputs(m, host_g, host_layers)
    seq = orc.Seq(om, prompt_tokens + max_steps * D + D)
    t0 = time.perf_counter()
    seq.prefill(prompt[:prompt_tokens])
    t_pre = time.perf_counter() - t0
    acc, t_steps, n_steps = 0, 0.0, 0
    while n_steps < max_steps and (n_steps < 2 or t_steps < budget_s):
        t0 = time.perf_counter()
        _, _, _, g = seq.step(D, tau, want_logits=False)
        seq.commit()
        t_steps += time.perf_counter() - t0
        acc += g
        n_steps += 1
    return {"value": acc / t_steps, "unit": "accepted tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"sequence 0 truncated to its first {prompt_tokens} prompt tokens, {n_steps} decode steps, all "
                      f"{m.n_layers} layers and the full vocabulary; the oracle decodes one sequence at a time, so its rate "
                      f"does not grow with the batch (prefill of the sample took {t_pre:.1f} s, not counted). The short "
                      f"context is the bound on the sample, not a shortcut that matters: an oracle step is {D + 1} rows through "
                      f"every weight matrix ({2 * (D + 1) * weight_params(m) / 1e9:.0f} GFLOP) plus attention over the context "
                      f"({4 * (D + 1) * m.n_layers * m.n_q_heads * m.head_dim * ctx_tokens / 1e9:.1f} GFLOP at the workload's mean "
                      f"context of {ctx_tokens:.0f} tokens), so by operation count its step at that context would be about "
                      f"{100 * 2 * m.n_layers * m.n_q_heads * m.head_dim * ctx_tokens / weight_params(m):.0f} % slower (an extrapolation, "
                      f"not a measurement)",
            "ms_per_step_per_sequence": 1e3 * t_steps / n_steps}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build measures the block-decode step on ONE GPU; --gpus %d is not supported "
              "(sequences are independent: more GPUs would each take a share of the batch)" % a.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2509_24007_amd import inputs as syn
    from paper_2509_24007_amd import sdlm

    wl = syn.workloads()[a.config]
    m, r = wl.model, wl.run
    if a.block_causal:
        m = dataclasses.replace(m, block_causal=True)
    tau = a.tau if a.tau is not None else r.tau
    taus = [tau] + ([t for t in (r.taus or []) if t != tau] if a.sweep else [])
    B, D = r.batch, r.block_D
    prompts = [p.numpy() for p in syn.make_prompts(wl.seed, B, r.prompt_lo, r.prompt_hi, m.vocab)]
    table_steps = 0 if (a.profile_all or a.phases == "main" or a.verify is not None) else min(32, a.steps)
    total_steps = a.warmup + a.steps + table_steps
    max_len = max(len(p) for p in prompts) + total_steps * D + D
    n_pages = sum((len(p) + total_steps * D + D + 15) // 16 + 1 for p in prompts) if r.paged else 0
    ceiling = copy_ceiling()
    side = torch.cuda.Stream() if a.graph else None
    with torch.cuda.stream(side):
        ctx = sdlm.Context(sdlm.model_cfg(m), max_batch=B, max_seq_len=max_len, block_D=D, tau=tau, paged=r.paged,
                           n_pages=n_pages, prefill_rows=a.prefill_rows, conf_fn=a.conf_fn, accept_rule=a.accept_rule)
    torch.cuda.synchronize()
    if a.graph:
        ctx.graph(True)
    want_cpu = not a.no_cpu_baseline
    t0 = time.perf_counter()
    host_g, host_layers = build_model(ctx, m, wl.seed, keep_host_layers=m.n_layers if want_cpu else None)
    t_build = time.perf_counter() - t0
    prof = True if a.profile_all else {"main": MAIN_PHASES, "none": None}.get(a.phases, tuple(a.phases.split(",")))
    if a.verify is not None:
        prof = None
    esz = 4 if m.dtype == "fp32" else 2
    results = []
    for ti, tv in enumerate(taus):
        if ti > 0:
            ctx.close()
            with torch.cuda.stream(side):
                ctx = sdlm.Context(sdlm.model_cfg(m), max_batch=B, max_seq_len=max_len, block_D=D, tau=tv, paged=r.paged, n_pages=n_pages,
                                   prefill_rows=a.prefill_rows, conf_fn=a.conf_fn, accept_rule=a.accept_rule)
            torch.cuda.synchronize()
            if a.graph:
                ctx.graph(True)
            build_model(ctx, m, wl.seed)
        t0 = time.perf_counter()
        dt, cnt, phases, n_end, tphases = run_tau(ctx, m, r, prompts, ti, a.steps, a.warmup, prof, table_steps if ti == 0 else 0, a.verify, a.force_accept, a.profile_every)
        t_total = time.perf_counter() - t0
        if a.force_accept:
            cnt = torch.full_like(cnt, a.force_accept)
        timed = cnt[a.warmup:a.warmup + a.steps].numpy().astype(np.int64)
        accepted = int(timed.sum())
        hist = np.bincount(timed.ravel(), minlength=D + 1)[1:].tolist()
        # context length of every sequence at every timed step (prompt + everything accepted before the step)
        lens0 = np.array([len(p) for p in prompts], dtype=np.int64)
        before = lens0[None, :] + np.concatenate([np.zeros((1, B), np.int64), np.cumsum(cnt.numpy().astype(np.int64), 0)[:-1]], 0)
        ctx_timed = before[a.warmup:a.warmup + a.steps]
        pend = np.concatenate([np.zeros((1, B), np.int64), cnt.numpy().astype(np.int64)[:-1]], 0)[a.warmup:a.warmup + a.steps]
        R_mean = float((pend + D).sum(1).mean())
        w_bytes, kv_bytes = algorithmic_bytes(m, esz, float(ctx_timed.sum(1).mean()), R_mean)
        lat = np.sort(np.array(run_tau.step_ms))
        results.append(dict(tau=tv, dt=dt, lat=lat, accepted=accepted, hist=hist, phases=phases, tphases=tphases, R_mean=R_mean,
                            w_bytes=w_bytes, kv_bytes=kv_bytes, ctx_mean=float(ctx_timed.mean()), t_total=t_total))
    main_r = results[0]
    ms_per_step = 1e3 * main_r["dt"] / a.steps
    # per-kernel accounting (per launch = one layer's kernel, or the LM head)
    d, h, F, V, L = m.head_dim, m.hidden, m.ffn, m.vocab, m.n_layers
    nq, nk = m.n_q_heads * d, m.n_kv_heads * d
    Rm = main_r["R_mean"]
    kv_layer = main_r["kv_bytes"] / L
    kern = {
        "attn": dict(bytes=kv_layer + 2 * Rm * nq * esz, flops=0.0),
        "qkv": dict(bytes=(nq + 2 * nk) * h * esz, flops=2.0 * Rm * (nq + 2 * nk) * h),
        "oproj": dict(bytes=h * nq * esz, flops=2.0 * Rm * h * nq),
        "gateup": dict(bytes=2 * F * h * esz, flops=4.0 * Rm * F * h),
        "down": dict(bytes=F * h * esz, flops=2.0 * Rm * F * h),
        "lmhead": dict(bytes=V * h * esz, flops=2.0 * B * D * V * h),
        "attn_merge": dict(bytes=0.0, flops=0.0),     # the split-KV partials: no algorithmic bytes of its own
    }
    # attention flops: 4 * d per (query row, head, visible key); rows of a sequence see about its context
    kern["attn"]["flops"] = 4.0 * d * m.n_q_heads * float(((main_r["ctx_mean"]) * Rm))
    table = {}
    for name, k in kern.items():
        ms, launches = main_r["phases"].get(name, (0.0, 0))
        src = "timed region"
        if launches == 0:
            ms, launches = main_r["tphases"].get(name, (0.0, 0))
            src = "extra steps after the timed region"
        if launches == 0:
            continue
        avg = ms / launches
        t_hbm = k["bytes"] / (PEAK_HBM_GBS * 1e9)
        t_mfma = k["flops"] / (PEAK_BF16_TFLOPS * 1e12)
        table[name] = dict(ms_total=ms, launches=launches, avg_us=1e3 * avg, gbs=k["bytes"] / (avg * 1e-3) / 1e9,
                           tflops=k["flops"] / (avg * 1e-3) / 1e12, bound="hbm" if t_hbm >= t_mfma or m.dtype == "fp32" else "mfma",
                           per_step_ms=ms / launches * (1 if name == "lmhead" else L), events=src)
    roof = None
    if table:
        # the dominant kernel is taken among the phases bracketed inside the timed region (default: the gate/up GEMM, the
        # longest kernel of the step in the rocprofv3 trace of the bf16 workloads); the extra-step figures of the other
        # phases carry the overhead of seven event pairs per layer and are for orientation only
        timed_names = [k for k in table if table[k]["events"] == "timed region"]
        dom = max(timed_names or list(table), key=lambda k: table[k]["per_step_ms"])
        t = table[dom]
        if t["bound"] == "hbm":
            roof = dict(kernel=dom, bound="hbm", achieved=t["gbs"], peak=PEAK_HBM_GBS, unit="GB/s", frac=t["gbs"] / PEAK_HBM_GBS, traffic=None)
        else:
            roof = dict(kernel=dom, bound="mfma", achieved=t["tflops"], peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=t["tflops"] / PEAK_BF16_TFLOPS, traffic=None)
        roof["traffic"] = measured_traffic(a.config, dom)
        if roof["bound"] == "hbm":
            roof["frac_of_copy_ceiling"] = t["gbs"] / ceiling["GBs"]
        roof["avg_launch_us"] = t["avg_us"]
        roof["launches"] = t["launches"]
        roof["sampled_every"] = a.profile_every if t["events"] == "timed region" else 1
        roof["events"] = t["events"]
    step_bytes = main_r["w_bytes"] + main_r["kv_bytes"]
    out = {
        "metric": "accepted tokens/sec and block-step latency; achieved HBM GB/s vs peak",
        "value": main_r["accepted"] / main_r["dt"],
        "unit": "accepted tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step,
        "step_latency_ms": {"median": float(np.median(main_r["lat"])), "p10": float(np.percentile(main_r["lat"], 10)),
                            "p90": float(np.percentile(main_r["lat"], 90)), "min": float(main_r["lat"][0]),
                            "max": float(main_r["lat"][-1]),
                            "note": "device time between per-step events on the library's stream, timed steps only; the "
                                    "context grows by the accepted tokens each step"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if m.dtype == "fp32" else "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name, "batch": B, "block_D": D, "tau": main_r["tau"], "paged_kv": bool(r.paged),
                   "prompt_len": [r.prompt_lo, r.prompt_hi], "kernels": ctx.kernel_info, "graph_replay": bool(a.graph),
                   "conf_fn": a.conf_fn, "accept_rule": a.accept_rule, "block_causal": bool(a.block_causal),
                   **({"forced_accept_per_step": a.force_accept} if a.force_accept else {}),
                   "decoding": "greedy longest-prefix (gamma_tau)" if a.verify is None else
                               "self-speculative (gamma_verify, rule %d): a step is the block step plus the verification pass" % a.verify},
        "gamma_hist": main_r["hist"],
        "tokens_per_step_per_seq": main_r["accepted"] / (a.steps * B),
        "rows_per_step": main_r["R_mean"],
        "mean_context": main_r["ctx_mean"],
        "step_algorithmic_GB": step_bytes / 1e9,
        "step_hbm_GBs": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "hbm_copy_ceiling": ceiling,
        "step_hbm_frac_of_copy_ceiling": step_bytes / (ms_per_step * 1e-3) / 1e9 / ceiling["GBs"],
        "roofline": roof,
        "kernels": {k: {kk: (round(vv, 3) if isinstance(vv, float) else vv) for kk, vv in v.items()} for k, v in table.items()},
        "prefill": {"prompt_tokens": int(sum(len(p) for p in prompts)), "seconds": round(run_tau.prefill_s, 3),
                    "tokens_per_s": sum(len(p) for p in prompts) / run_tau.prefill_s,
                    "note": "causal pass over the prompts through the same kernels (pending-row path), LM head skipped; "
                            "prompts come from host memory; last tau's run when sweeping"},
        "setup_s": {"weights": round(t_build, 1), "prefill_and_run": round(main_r["t_total"], 1)},
    }
    if a.verify is not None:    # the byte accounting above describes the block step alone
        for k in ("step_algorithmic_GB", "step_hbm_GBs", "step_hbm_frac", "step_hbm_frac_of_copy_ceiling", "roofline"):
            out[k] = None
        out["verify_rows_per_step"] = B * ((D - 2) + (D - 1) * D)
    if len(results) > 1:
        out["tau_sweep"] = [dict(tau=x["tau"], value=x["accepted"] / x["dt"], ms_per_step=1e3 * x["dt"] / a.steps,
                                 gamma_hist=x["hist"]) for x in results]
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    if want_cpu:
        out["cpu_baseline"] = cpu_baseline(m, host_g, host_layers, prompts[0], D, tau, prompt_tokens=min(8, len(prompts[0])),
                                           ctx_tokens=main_r["ctx_mean"])
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
