#!/usr/bin/env python3
"""Benchmark of the RSD hot path on one MI355X.

A "step" is one full pass of Algorithm 1 over one batch of synthetic prompts:
every reasoning step runs draft decode, reward-model scoring, the delta gate
with rollback and target regeneration, until max_steps.  The default workload
is configuration 1 (bf16, batch 1, 1.5B draft / 7B target / 1.5B reward model,
256-token prompt, 16 steps of <= 64 tokens, top-p 0.95 at T = 0.7, delta 0.7).
Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
PROBE_OPS = {"qkv": 0, "o": 1, "gate_up": 2, "down": 3, "head": 4}


def cpu_baseline(w, budget_s=20.0):
    """The fp64 CPU checker timed on a bounded sample of the same workload:
    the three models at full width and vocabulary (full depth if the host has
    the memory, else 12 layers each), one sequence, the first two reasoning steps
    capped at 8 tokens."""
    import numpy as np
    import torch
    from dataclasses import replace
    from rsd_inputs import workload, model_weights_np, prompt_tokens, prompt_lengths, uniforms
    from oracle import rsd_oracle as O

    # full depth where the host can hold the models twice over (fp32 as generated + the checker's fp64
    # copies: about 130 GB for cfg1); 12 layers otherwise
    layers = 12
    try:
        import psutil
        if psutil.virtual_memory().available > 200e9:
            layers = w.draft.n_layers
    except ImportError:
        pass
    ws = workload(w.name, n_layers=layers, batch=1, step_cap=8, max_steps=2)
    cores = min(16, os.cpu_count() or 1)
    models = [O.OracleModel(s, model_weights_np(ws.seed, i, s, threads=cores)) for i, s in enumerate(ws.shapes)]
    toks, lens = prompt_tokens(ws), prompt_lengths(ws)
    P = O.Params(delta=ws.delta, sep_id=ws.sep_id, step_cap=ws.step_cap, max_steps=ws.max_steps, max_ctx=ws.max_ctx,
                 temperature=float(np.float32(ws.temperature)), top_p=float(np.float32(ws.top_p)))
    t0 = time.time()
    out = O.generate_sequence(models[0], models[1], models[2], toks[0, :lens[0]],
                              uniforms(ws, "U_DRAFT", ws.max_ctx)[0], uniforms(ws, "U_TARGET", ws.max_ctx)[0],
                              uniforms(ws, "U_GATE", ws.max_steps)[0], P)
    dt = time.time() - t0
    n = len(out["tokens"]) - int(lens[0])
    return {"value": n / dt, "unit": "tokens/s", "cores": int(torch.get_num_threads()), "kind": "oracle",
            "sample": f"{ws.name} shapes at full width and vocabulary, {layers} of {w.draft.n_layers} layers per model, "
                      f"1 sequence, prompt {int(lens[0])} tokens + the first {ws.max_steps} reasoning steps of <= {ws.step_cap} tokens ({n} tokens) "
                      f"(prompt prefill of all touched models included), {dt:.1f} s"
                      + ("" if layers == w.draft.n_layers else
                         f"; at full depth the rate is roughly {w.draft.n_layers / layers:.1f}x lower")}


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "cfg1_target_gate_up_hbm_traffic.txt")
KERNEL_SOURCES = ("paper_2501_19324_amd/csrc/gemv.cuh", "paper_2501_19324_amd/csrc/common.cuh")


def measured_traffic():
    """HBM bytes per launch of the probed kernel from the hardware counters recorded in
    profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy kernel), or None when no
    record exists or the kernel's sources have changed since it was taken."""
    import hashlib
    try:
        rec = dict(line.strip().split("=", 1) for line in open(TRAFFIC_FILE) if "=" in line and " " not in line.strip())
        h = hashlib.sha256()
        for p in KERNEL_SOURCES:
            h.update(open(os.path.join(ROOT, p), "rb").read())
        if rec.get("kernel_source_sha256") != h.hexdigest():
            return None
        return int(rec["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--delta", type=float, default=None)
    ap.add_argument("--layers", type=int, default=None, help="reduce depth (debugging only; invalid as a result)")
    ap.add_argument("--probe", default="gate_up", choices=sorted(PROBE_OPS))
    ap.add_argument("--probe-model", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graphs", action="store_true")
    ap.add_argument("--max-steps", type=int, default=0, help="stop each pass after this many reasoning steps (debugging)")
    ap.add_argument("--kv-pool-gb", default="", help="KV pool sizes in GB for draft,target,PRM (default: worst case)")
    ap.add_argument("--ops", action="store_true", help="extra passes after the timed region: per-projection table")
    ap.add_argument("--merge", default="none", choices=["none", "draft", "target"],
                    help="reward head on the draft's or the target's trunk instead of a third model (not the headline workload)")
    ap.add_argument("--sd-k", type=int, default=0,
                    help="regenerate rejected steps by speculative decoding with this many proposals per round "
                         "(greedy workloads only; not the headline workload)")
    ap.add_argument("--greedy", action="store_true", help="override the workload's sampler with greedy decoding "
                                                          "(the paper's default setting; needed by --sd-k on cfg1)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="before the timed region run a plain 256 MiB device copy kernel three times (reference "
                         "point for scaling hardware traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (sequences are independent; more GPUs would shard the "
              "batch with no communication); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from rsd_inputs import workload
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session

    kw = {}
    if args.layers:
        kw["n_layers"] = args.layers
    if args.greedy:
        kw.update(temperature=0.0, top_p=1.0)
    w = workload(args.workload, **kw)
    merge = {"none": 0, "draft": 1, "target": 2}[args.merge]
    if merge:
        from dataclasses import replace
        w = replace(w, prm=replace(w.draft if merge == 1 else w.target, head_kind="reward"))
    delta = w.delta if args.delta is None else args.delta
    t_setup = time.time()
    pools = tuple(int(float(x) * 1e9) for x in args.kv_pool_gb.split(",")) if args.kv_pool_gb else (0, 0, 0)
    s = Session(w, delta=delta, use_graphs=0 if args.no_graphs else 1, kv_pool_bytes=pools, merge_prm=merge, sd_k=args.sd_k)
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    first = dict(ms=0.0, tokens=0)       # the first reasoning step (it holds the prompt prefills), summed over the timed passes

    def one_pass():
        s.reset()
        try:
            # Algorithm 1's loop in two calls, so that the first step can be told apart from the steady state
            t_first = time.perf_counter()
            g1 = R.rsd_generate(s.ctx, max_steps=1, want_tokens=False)
            first["ms"] += (time.perf_counter() - t_first) * 1e3
            first["tokens"] += g1["n_committed"]
            if args.max_steps == 1 or (g1["finished"] != 0).all():
                return g1
            g = R.rsd_generate(s.ctx, max_steps=args.max_steps, want_tokens=False)
            for k in ("n_draft", "n_target", "n_accept", "n_reject", "n_sd_rounds", "n_sd_proposed", "n_sd_kept"):
                g[k] += g1[k]
            return g
        except R.RsdError as e:
            if e.code != R.RSD_ENOMEM:
                raise
            # KV pool exhausted: a clean stop; report what was generated until then
            st = R.rsd_export_state(s.ctx, want_tokens=False)
            print(f"# KV pool exhausted: {e}; contexts reached {int(st['ctx_len'].min())}..{int(st['ctx_len'].max())}",
                  file=sys.stderr)
            return dict(n_committed=int((st["ctx_len"] - s.prompt_len).sum()), n_draft=0, n_target=0, n_accept=0,
                        n_reject=0)

    if args.calib_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)       # one elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        one_pass()
    first.update(ms=0.0, tokens=0)
    R.rsd_stage_ms(s.ctx, reset=True)
    R.rsd_probe_start(s.ctx, args.probe_model, PROBE_OPS[args.probe], 8192, 4)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tokens = drafted = targeted = acc = rej = 0
    sd = dict(rounds=0, proposed=0, kept=0)
    for _ in range(args.steps):
        g = one_pass()
        tokens += g["n_committed"]; drafted += g["n_draft"]; targeted += g["n_target"]
        acc += g["n_accept"]; rej += g["n_reject"]
        for k in sd:
            sd[k] += g.get("n_sd_" + k, 0)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    probe = R.rsd_probe_read(s.ctx)
    stage = R.rsd_stage_ms(s.ctx)

    roof = None
    traffic = measured_traffic() if (args.workload == "cfg1" and args.probe == "gate_up" and args.probe_model == 1
                                     and not args.layers) else None
    if probe["n"] > 0:
        avg_s = probe["total_ms"] / probe["n"] * 1e-3
        gbs = probe["bytes_per_launch"] / avg_s / 1e9
        roof = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                "kernel": f"gemv_flat_kernel ({args.probe} projection of model {args.probe_model}, single-token decode)",
                "bytes_per_launch": probe["bytes_per_launch"], "avg_launch_us": round(avg_s * 1e6, 2),
                "launches_timed": probe["n"]}
    # decode-stage view of the same roofline: bytes every sampled token has to read
    dec_bytes = drafted * w.draft.decode_weight_bytes() + targeted * w.target.decode_weight_bytes()
    dec_s = (stage[0] + stage[3]) * 1e-3
    line = {
        "metric": "generated tokens/s (1 GPU) per delta",
        "value": round(tokens / dt, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.draft.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, draft {w.draft.n_layers}L-d{w.draft.d_model}, target "
                               f"{w.target.n_layers}L-d{w.target.d_model}, PRM {w.prm.n_layers}L-d{w.prm.d_model}, "
                               f"vocab {w.draft.vocab}, prompts {w.prompt_len_min}-{w.prompt_len_max}, "
                               f"{w.max_steps} steps x <= {w.step_cap} tokens, T={w.temperature}, top_p={w.top_p}",
                   "delta": delta, "merge_prm": args.merge, "committed_tokens_per_pass": tokens // max(args.steps, 1),
                   "accept_rate": round(acc / max(acc + rej, 1), 4), "draft_tokens": drafted, "target_tokens": targeted,
                   "stage_ms_per_pass": {k: round(v / args.steps, 2) for k, v in zip(("draft", "prm", "gate", "target"), stage)},
                   # (with speculative regeneration the target stage also holds draft proposals and chunked passes)
                   "decode_weight_stream_GBs": round(dec_bytes / dec_s / 1e9, 1) if dec_s > 0 and not args.sd_k else None,
                   # generation after the first step (which holds the prompt prefills of the models it touches)
                   "steady_state_tokens_per_s": round((tokens - first["tokens"]) / (dt - first["ms"] * 1e-3), 2)
                   if tokens > first["tokens"] and dt > first["ms"] * 1e-3 else None,
                   "first_step_ms_per_pass": round(first["ms"] / max(args.steps, 1), 2),
                   "mean_step_tokens": round(tokens / max(acc + rej, 1), 2),
                   "target_token_fraction": round(targeted / max(tokens, 1), 4),
                   # forward cost by the rule of 2 x parameters per token (Section 3, "Computation Analysis"; the reward model is counted): draft tokens through
                   # the draft, the same tokens through the reward model, target tokens through the target; against
                   # every committed token through the target alone
                   "flops_2N": {"rsd": 2.0 * (drafted * (w.draft.n_params() + w.prm.n_params()) + targeted * w.target.n_params()),
                                "target_only": 2.0 * tokens * w.target.n_params()},
                   "setup_s": round(t_setup, 1)},
        "roofline": roof,
    }
    if args.sd_k:
        line["config"]["sd_k"] = args.sd_k
        line["config"]["sd"] = sd
    if args.ops:
        table = {}
        for model, shape in ((0, w.draft), (1, w.target)):
            for name, op in PROBE_OPS.items():
                R.rsd_probe_start(s.ctx, model, op, 4096, 1)
                one_pass()
                p = R.rsd_probe_read(s.ctx)
                if p["n"]:
                    us = p["total_ms"] / p["n"] * 1e3
                    table[f"m{model}.{name}"] = {"us": round(us, 2), "MB": round(p["bytes_per_launch"] / 1e6, 2),
                                                 "GBs": round(p["bytes_per_launch"] / us / 1e3, 1), "n": p["n"]}
        line["config"]["ops"] = table
    s.close()
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
