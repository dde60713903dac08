#!/usr/bin/env python3
"""Benchmark of the RSD hot path on one MI355X.

A "step" is one reasoning step of Algorithm 1 for the whole batch (one call of
rsd_step: draft decode of the step, reward-model scoring, the delta gate with
rollback, target regeneration of the rejected sequences); when every sequence
of the batch has run its steps the prompts are set again and the next pass
begins.  The default workload is the largest configuration that fits one GPU:
configuration 3 (bf16, batch 16, 1.5B draft / 72B target / 7B reward model all
resident, 512-token prompts, 16 steps of <= 128 tokens, greedy, delta 0.7).

After the timed region the same process measures, as sub-records of the one
JSON line it prints: configuration 2 (batch 64) for every delta of its sweep,
configuration 1 (batch 1) and configuration 4 (batch 256, long context) for a
few steps each, and the fp64 CPU checker on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PROBE_OPS = {"qkv": 0, "o": 1, "gate_up": 2, "down": 3, "head": 4}
DECODE, PREFILL = 0, 1


def cpu_baseline(w, budget_layers=None):
    """The fp64 CPU checker timed on a bounded sample of the same workload: the three
    models at full width and vocabulary, as many layers of each as the host's memory
    holds in fp64, one sequence, its prompt and the first reasoning steps cut short."""
    import numpy as np
    from rsd_inputs import workload, model_weights_np, prompt_tokens, prompt_lengths, uniforms
    from oracle import rsd_oracle as O

    # fp64 bytes of one model = 8 x parameters (plus the fp32 copy it is generated in): full depth when
    # the three models fit in about half of the free memory, else the same number of layers for each
    avail = 64e9
    try:
        import psutil
        avail = psutil.virtual_memory().available
    except ImportError:
        pass
    avail = min(avail, 240e9)            # stay well inside the box's per-command limit
    full = [s.n_layers for s in w.shapes]

    def need(layers):
        tot = 0
        for s, L in zip(w.shapes, layers):
            per_layer = 2 * s.d_model * s.q_dim + 2 * s.d_model * s.kv_dim + 3 * s.d_model * s.d_ffn
            tot += (L * per_layer + 2 * s.vocab * s.d_model) * 12
        return tot
    layers = list(full)
    if budget_layers or need(layers) > 0.5 * avail:      # (the 72B target alone is 580 GB in fp64)
        layers = [min(L, budget_layers or 4) for L in full]
        while max(layers) > 1 and need(layers) > 0.5 * avail:
            layers = [max(1, L - 1) for L in layers]
    L = max(layers)
    step_cap, max_steps, n_seq = 16, 6, 2
    ws = workload(w.name, n_layers=L, batch=n_seq, step_cap=step_cap, max_steps=max_steps)
    threads = min(16, os.cpu_count() or 1)
    models = [O.OracleModel(s, model_weights_np(ws.seed, i, s, threads=threads)) for i, s in enumerate(ws.shapes)]
    progress("CPU checker: fp64 models generated")
    toks, lens = prompt_tokens(ws), prompt_lengths(ws)
    P = O.Params(delta=ws.delta, sep_id=ws.sep_id, step_cap=ws.step_cap, max_steps=ws.max_steps, max_ctx=ws.max_ctx,
                 temperature=float(np.float32(ws.temperature)), top_p=float(np.float32(ws.top_p)))
    cores = blas_threads()
    ud, ut, ug = uniforms(ws, "U_DRAFT", ws.max_ctx), uniforms(ws, "U_TARGET", ws.max_ctx), uniforms(ws, "U_GATE", ws.max_steps)
    t0 = time.time()
    n = 0
    for b in range(n_seq):
        out = O.generate_sequence(models[0], models[1], models[2], toks[b, :lens[b]], ud[b], ut[b], ug[b], P)
        n += len(out["tokens"]) - int(lens[b])
        progress(f"CPU checker: sequence {b + 1} of {n_seq} done")
    dt = time.time() - t0
    used = [min(f, L) for f in full]
    scale = ""
    if used != full:
        scale = ("; layers timed per model (draft, target, reward) " + "/".join(map(str, used)) + " of " + "/".join(map(str, full))
                 + ": the layer part of the cost grows in proportion, so at full depth the rate is roughly "
                 + f"{max(f / u for f, u in zip(full, used)):.0f}x lower for the deepest model")
    return {"value": n / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{ws.name} shapes at full width and vocabulary, {n_seq} sequences one after the other, prompt {int(lens[0])} tokens + the first "
                      f"{ws.max_steps} reasoning steps of <= {ws.step_cap} tokens ({n} tokens; prompt prefill of all touched "
                      f"models included), {dt:.1f} s" + scale}


def progress(msg):
    """One line on stderr (stdout carries the single JSON record): a run of several minutes shows where it is."""
    print(f"# [{time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def blas_threads():
    """Threads the checker's NumPy matrix products actually run on."""
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads", 0) for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return int(max(n))
    except Exception:
        pass
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))


def kernel_sources_sha():
    import hashlib
    h = hashlib.sha256()
    for p in ("paper_2501_19324_amd/csrc/gemm.h", "paper_2501_19324_amd/csrc/gemv.h", "paper_2501_19324_amd/csrc/common.h"):
        h.update(open(os.path.join(ROOT, p), "rb").read())
    return h.hexdigest()


def measured_traffic(name):
    """HBM bytes per launch of the probed kernel from the hardware counters recorded in
    profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy kernel), or None when no
    record exists or the kernel's sources have changed since it was taken."""
    try:
        path = os.path.join(ROOT, "profiles", f"{name}_target_gate_up_hbm_traffic.txt")
        rec = dict(line.strip().split("=", 1) for line in open(path) if "=" in line and " " not in line.strip())
        if rec.get("kernel_source_sha256") != kernel_sources_sha():
            return None
        return int(rec["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


class Runner:
    """Steps a Session: rsd_step after rsd_step, setting the prompts again when a pass is over."""

    def __init__(self, R, s):
        self.R, self.s = R, s
        self.left = 0           # sequences still running in the current pass
        self.exhausted = None
        self.tot = dict(steps=0, tokens=0, drafted=0, targeted=0, acc=0, rej=0, passes=0)
        self.touched = None     # sequences of the current pass for which the target has generated a step
        self.pass_log = []      # per pass: [index of its last step so far, sequences, sequences the target never served]

    def step(self):
        import numpy as np
        R, s = self.R, self.s
        if self.left == 0:
            s.reset()
            self.running = np.ones(s.w.batch, bool)
            self.touched = np.zeros(s.w.batch, bool)
            self.tot["passes"] += 1
            self.pass_log.append([0, s.w.batch, s.w.batch])
        o = R.rsd_step(s.ctx)
        live = self.running
        t = self.tot
        t["steps"] += 1
        t["tokens"] += int(o["final_len"][live].sum())
        t["drafted"] += int(o["draft_len"][live].sum())
        acc = o["accepted"][live] != 0
        t["acc"] += int(acc.sum())
        t["rej"] += int((~acc).sum())
        t["targeted"] += int(o["final_len"][live][~acc].sum())
        idx = np.flatnonzero(live)
        self.touched[idx[~acc]] = True
        self.pass_log[-1][0] = t["steps"]
        self.pass_log[-1][2] = int((~self.touched).sum())
        self.running = o["finished"] == 0
        self.left = int(self.running.sum())
        return o

    def snapshot(self):
        return dict(self.tot)

    def draft_only_fraction(self, since_step):
        """Share of sequences the target never generated a step for, over the passes that had a step after step
        `since_step` (a pass the window cuts counts with all the steps it has had so far)."""
        seen = [p for p in self.pass_log if p[0] > since_step]
        n = sum(p[1] for p in seen)
        return round(sum(p[2] for p in seen) / n, 4) if n else None


def iteration_record(R, s, shapes, reset=True):
    """Decode-loop view of the HBM roofline, per policy model: bytes one iteration has to move
    (the weights once, the keys/values every active sequence attends to, the new entries) over
    the GPU time of the decode loops."""
    out = {}
    for which, name in ((0, "draft"), (1, "target")):
        st = R.rsd_iter_stats(s.ctx, which, reset=reset)
        if st["iterations"] == 0 or st["gpu_ms"] <= 0:
            out[name] = None
            continue
        m = shapes[which]
        kvb = m.kv_bytes_per_token
        by = st["iterations"] * m.decode_weight_bytes() + (st["kv_tokens_read"] + st["seq_iterations"]) * kvb
        gbs = by / (st["gpu_ms"] * 1e-3) / 1e9
        out[name] = {"iterations": st["iterations"], "ms_per_iteration": round(st["gpu_ms"] / st["iterations"], 4),
                     "mean_active_sequences": round(st["seq_iterations"] / st["iterations"], 2),
                     "mean_rows_launched": round(st["row_iterations"] / st["iterations"], 2),
                     "mean_context": round(st["kv_tokens_read"] / max(st["seq_iterations"], 1), 1),
                     "GB_per_iteration": round(by / st["iterations"] / 1e9, 3),
                     "GBs": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                     "ms_per_token": round(st["gpu_ms"] / max(st["seq_iterations"], 1), 4)}
    return out


def probe_record(R, s, slot, kind):
    clk = R.rsd_probe_clock(s.ctx, slot) if kind == "mfma" else None
    p = R.rsd_probe_read(s.ctx, slot)
    if p["n"] == 0 or p["total_ms"] <= 0:
        return None
    sec = p["total_ms"] * 1e-3
    if kind == "hbm":
        gbs = p["total_bytes"] / sec / 1e9
        return {"launches_timed": p["n"], "avg_launch_us": round(sec / p["n"] * 1e6, 2),
                "bytes_per_launch": p["total_bytes"] // p["n"], "GBs": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4)}
    tf = p["total_flops"] / sec / 1e12
    rec = {"launches_timed": p["n"], "avg_launch_us": round(sec / p["n"] * 1e6, 2),
           "flops_per_launch": p["total_flops"] // p["n"], "TFLOPs": round(tf, 1),
           "frac_of_bf16_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)}
    if clk and clk["launches"] > 0 and clk["ref_ticks"] > 0:
        # shader clock read inside the probed launches (against the constant 100 MHz counter); the published
        # peak is quoted at 2400 MHz, so the second figure is the fraction of what the MFMA units can issue
        # at the clock the chip actually held
        mhz = clk["shader_ticks"] / clk["ref_ticks"] * 100.0
        rec["shader_clock_mhz"] = round(mhz, 1)
        rec["frac_of_mfma_peak_at_that_clock"] = round(tf / (MFMA_BF16_PEAK_TFLOPS * mhz / 2400.0), 4)
    return rec


def run_steps(R, s, w, n_steps, warmup=0, probes=True, probe_stride=8):
    """Warm up, then time n_steps reasoning steps; returns the record of the timed region."""
    import torch
    r = Runner(R, s)
    for i in range(warmup):
        r.step()
        progress(f"warm-up step {i + 1} of {warmup} done")
    base = r.snapshot()
    R.rsd_stage_ms(s.ctx, reset=True)
    for which in (0, 1):
        R.rsd_iter_stats(s.ctx, which, reset=True)
    if probes:
        R.rsd_probe_start(s.ctx, 0, 1, DECODE, PROBE_OPS["gate_up"], 8192, probe_stride)   # target gate/up, decode
        R.rsd_probe_start(s.ctx, 1, 2, PREFILL, PROBE_OPS["gate_up"], 8192, 1)             # reward model gate/up, scoring pass
        R.rsd_probe_start(s.ctx, 2, 2, PREFILL, PROBE_OPS["down"], 8192, 1)
        R.rsd_probe_start(s.ctx, 3, 0, DECODE, PROBE_OPS["gate_up"], 8192, probe_stride)   # draft gate/up, decode
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    first_ms, first_tok = 0.0, 0
    t_said = time.perf_counter()
    for i in range(n_steps):
        new_pass = r.left == 0
        ta = time.perf_counter()
        before = r.tot["tokens"]
        r.step()
        if new_pass:            # the first step of a pass holds the prompt prefills
            first_ms += (time.perf_counter() - ta) * 1e3
            first_tok += r.tot["tokens"] - before
        if time.perf_counter() - t_said > 20.0:       # (the step has ended on the host: rsd_step returns its records)
            t_said = time.perf_counter()
            progress(f"timed step {i + 1} of {n_steps} done")
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    t = {k: r.tot[k] - base[k] for k in base}
    stage = R.rsd_stage_ms(s.ctx)
    rec = {"seconds": dt, "tokens": t["tokens"], "tokens_per_s": round(t["tokens"] / dt, 2),
           "ms_per_step": round(dt / max(n_steps, 1) * 1e3, 2),
           "accept_rate": round(t["acc"] / max(t["acc"] + t["rej"], 1), 4),
           "draft_tokens": t["drafted"], "target_tokens": t["targeted"],
           "mean_step_tokens": round(t["tokens"] / max(t["acc"] + t["rej"], 1), 2),
           "target_token_fraction": round(t["targeted"] / max(t["tokens"], 1), 4),
           # sequences the target never had to generate a step for (Section 4 reports this share of questions)
           "draft_only_sequence_fraction": r.draft_only_fraction(base["steps"]),
           "stage_ms_per_step": {k: round(v / max(n_steps, 1), 2) for k, v in zip(("draft", "prm", "gate", "target"), stage)},
           "steps_after_first_tokens_per_s": round((t["tokens"] - first_tok) / (dt - first_ms * 1e-3), 2)
           if t["tokens"] > first_tok and dt > first_ms * 1e-3 else None,
           # forward cost by the rule of 2 x parameters per token (Section 3, "Computation Analysis"; the reward
           # model is counted): draft tokens through the draft and the reward model, target tokens through the
           # target; against every committed token through the target alone
           "flops_2N": {"rsd": 2.0 * (t["drafted"] * (w.draft.n_params() + w.prm.n_params()) + t["targeted"] * w.target.n_params()),
                        "target_only": 2.0 * t["tokens"] * w.target.n_params()},
           "iteration": iteration_record(R, s, w.shapes)}
    it = rec["iteration"]
    rec["draft_ms_per_token"] = it["draft"]["ms_per_token"] if it.get("draft") else None
    rec["target_ms_per_token"] = it["target"]["ms_per_token"] if it.get("target") else None
    rec["draft_ms_per_iteration"] = it["draft"]["ms_per_iteration"] if it.get("draft") else None
    rec["target_ms_per_iteration"] = it["target"]["ms_per_iteration"] if it.get("target") else None
    rec["prm_ms_per_step"] = rec["stage_ms_per_step"]["prm"]
    if probes:
        rec["probe_target_gate_up"] = probe_record(R, s, 0, "hbm")
        gu, dn = probe_record(R, s, 1, "mfma"), probe_record(R, s, 2, "mfma")
        rec["prm_prefill"] = {"gate_up_gemm": gu, "down_gemm": dn}
        rec["probe_draft_gate_up"] = probe_record(R, s, 3, "hbm")
    return rec


def workload_text(w):
    return (f"{w.name}: batch {w.batch}, draft {w.draft.n_layers}L-d{w.draft.d_model}, target "
            f"{w.target.n_layers}L-d{w.target.d_model}, PRM {w.prm.n_layers}L-d{w.prm.d_model}, vocab {w.draft.vocab}, "
            f"prompts {w.prompt_len_min}-{w.prompt_len_max}, {w.max_steps} steps x <= {w.step_cap} tokens, "
            f"T={w.temperature}, top_p={w.top_p}")


def slim(rec):
    """A sub-record without the bulky parts."""
    keep = ("tokens_per_s", "ms_per_step", "accept_rate", "mean_step_tokens", "target_token_fraction",
            "draft_only_sequence_fraction", "draft_ms_per_token",
            "target_ms_per_token", "draft_ms_per_iteration", "target_ms_per_iteration", "prm_ms_per_step",
            "steps_after_first_tokens_per_s", "tokens", "seconds")
    out = {k: rec[k] for k in keep if k in rec}
    out["seconds"] = round(out["seconds"], 2)
    out["iteration_frac_of_hbm_peak"] = {k: (v["frac_of_hbm_peak"] if v else None) for k, v in rec["iteration"].items()}
    if rec.get("prm_prefill") and rec["prm_prefill"].get("gate_up_gemm"):
        out["prm_gate_up_frac_of_mfma_peak"] = rec["prm_prefill"]["gate_up_gemm"]["frac_of_bf16_mfma_peak"]
    return out


def attention_probe(args):
    """Decode attention alone at given context lengths: bytes = sum of context x 2 x kv heads x head dim x 2
    per layer launch."""
    import numpy as np
    import torch
    from rsd_inputs import workload
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session

    kw = {"batch": args.batch} if args.batch else {}
    w = workload(args.workload, **kw)
    pools = tuple(int(float(x) * 1e9) for x in args.kv_pool_gb.split(",")) if args.kv_pool_gb else (0, 0, 0)
    s = Session(w, kv_pool_bytes=pools)
    rows = []
    for spec in args.contexts.split(","):
        if spec == "ragged":            # configuration 2's own prompt lengths plus half of its steps
            ctx = np.minimum(s.prompt_len + w.step_cap * w.max_steps // 2, w.max_ctx).astype(np.int32)
        else:
            ctx = np.full(w.batch, min(int(spec), w.max_ctx), np.int32)
        for which, name in ((0, "draft"), (1, "target")):
            m = w.shapes[which]
            try:
                ms = R.rsd_probe_attention(s.ctx, which, ctx, args.reps)
            except R.RsdError as e:
                rows.append({"model": name, "contexts": spec, "error": str(e)})
                continue
            by = int(ctx.sum()) * 2 * m.kv_dim * 2
            us = ms / args.reps * 1e3
            rows.append({"model": name, "contexts": spec, "batch": w.batch, "mean_context": float(ctx.mean()),
                         "bytes_per_launch": by, "avg_launch_us": round(us, 2), "GBs": round(by / us / 1e3, 1),
                         "frac_of_hbm_peak": round(by / us / 1e3 / HBM_PEAK_GBS, 4)})
    s.close()
    print(json.dumps({"probe": "decode attention (one layer launch; rotary embedding, cache write and split merge included)",
                      "workload": workload_text(w), "reps": args.reps, "rows": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--delta", type=float, default=None)
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch (configuration 4 at 192 sequences)")
    ap.add_argument("--layers", type=int, default=None, help="reduce depth (debugging only; invalid as a result)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the sub-records of the other configurations")
    ap.add_argument("--no-graphs", action="store_true")
    ap.add_argument("--no-probes", action="store_true")
    ap.add_argument("--kv-pool-gb", default="", help="KV pool sizes in GB for draft,target,PRM (default: worst case)")
    ap.add_argument("--until-enomem", action="store_true",
                    help="one pass only; a KV pool that runs out ends the run cleanly and the context reached is reported")
    ap.add_argument("--merge", default="none", choices=["none", "draft", "target"],
                    help="reward head on the draft's or the target's trunk instead of a third model (not the headline workload)")
    ap.add_argument("--sd-k", type=int, default=0,
                    help="regenerate rejected steps by speculative decoding with this many proposals per round")
    ap.add_argument("--greedy", action="store_true", help="override the workload's sampler with greedy decoding")
    ap.add_argument("--calib-copy", action="store_true",
                    help="before the timed region run a plain 256 MiB device copy kernel three times (reference "
                         "point for scaling hardware traffic counters)")
    ap.add_argument("--probe", default="", choices=["", "attention"], help="attention: time the decode attention kernel alone")
    ap.add_argument("--contexts", default="1024,4096,8192", help="--probe attention: context lengths (or 'ragged')")
    ap.add_argument("--reps", type=int, default=200)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on exactly one GPU (sequences are independent; more GPUs would shard the "
              "batch with no communication); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.probe == "attention":
        attention_probe(args)
        return

    import numpy as np
    import torch
    from dataclasses import replace
    from rsd_inputs import workload
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session

    kw = {}
    if args.layers:
        kw["n_layers"] = args.layers
    if args.greedy:
        kw.update(temperature=0.0, top_p=1.0)
    if args.batch:
        kw["batch"] = args.batch
    w = workload(args.workload, **kw)
    merge = {"none": 0, "draft": 1, "target": 2}[args.merge]
    if merge:
        w = replace(w, prm=replace(w.draft if merge == 1 else w.target, head_kind="reward"))
    delta = w.delta if args.delta is None else args.delta
    progress(f"{w.name}: generating weights and creating the context")
    t_setup = time.time()
    pools = tuple(int(float(x) * 1e9) for x in args.kv_pool_gb.split(",")) if args.kv_pool_gb else (0, 0, 0)
    s = Session(w, delta=delta, use_graphs=0 if args.no_graphs else 1, kv_pool_bytes=pools, merge_prm=merge, sd_k=args.sd_k)
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup
    progress(f"set up in {t_setup:.1f} s; stepping")

    if args.calib_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)       # one elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    note = None
    if args.until_enomem:
        # one pass, step by step, until the steps or the pool run out
        r = Runner(R, s)
        R.rsd_stage_ms(s.ctx, reset=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        per_step = []
        try:
            for i in range(w.max_steps):
                ta = time.perf_counter()
                before = r.tot["tokens"]
                r.step()
                per_step.append((round((time.perf_counter() - ta) * 1e3, 1), r.tot["tokens"] - before))
                print(f"# step {i + 1}: {per_step[-1][0]} ms, {per_step[-1][1]} tokens", file=sys.stderr, flush=True)
                if r.left == 0:
                    break
        except R.RsdError as e:
            if e.code != R.RSD_ENOMEM:
                raise
            note = f"KV pool exhausted after {len(per_step)} steps: {e}"
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        st = R.rsd_export_state(s.ctx, want_tokens=False)
        t = r.tot
        rec = {"seconds": dt, "tokens": t["tokens"], "tokens_per_s": round(t["tokens"] / dt, 2),
               "ms_per_step": round(dt / max(len(per_step), 1) * 1e3, 2),
               "accept_rate": round(t["acc"] / max(t["acc"] + t["rej"], 1), 4),
               "draft_only_sequence_fraction": r.draft_only_fraction(0),
               "steps_run": len(per_step), "note": note,
               "context_reached": [int(st["ctx_len"].min()), int(st["ctx_len"].max())],
               "kv_len_reached": {n: [int(st["kv_len"][i].min()), int(st["kv_len"][i].max())] for i, n in enumerate(("draft", "target", "prm"))},
               "stage_ms_per_step": {k: round(v / max(len(per_step), 1), 2) for k, v in zip(("draft", "prm", "gate", "target"), R.rsd_stage_ms(s.ctx))},
               "per_step_ms_tokens": per_step, "iteration": iteration_record(R, s, w.shapes)}
        steps_timed = len(per_step)
    else:
        rec = run_steps(R, s, w, args.steps, args.warmup, probes=not args.no_probes)
        steps_timed = args.steps

    roof = None
    pr = rec.get("probe_target_gate_up")
    if pr:
        tgt = w.shapes[1]
        even = (2 * tgt.d_ffn + 255) // 256 >= 200       # the library's rule for the evenly dealt few-row GEMM
        kern = ("gemv_flat_kernel" if w.batch == 1 else "gemm_tile_kernel" if w.batch > 64
                else "gemm_rows_sk_kernel" if even else "gemm_rows_kernel")
        roof = {"bound": "hbm", "achieved": pr["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": pr["frac"],
                "traffic": measured_traffic(w.name) if not (args.layers or args.batch) else None,
                "kernel": f"{kern} (gate+up projection of the target model, decode iteration of {w.batch} row(s))",
                "bytes_per_launch": pr["bytes_per_launch"], "avg_launch_us": pr["avg_launch_us"],
                "launches_timed": pr["launches_timed"],
                # the same roofline for the whole decode iteration (all kernels, launch gaps included)
                "iteration_frac": {k: (v["frac_of_hbm_peak"] if v else None) for k, v in rec["iteration"].items()}}
    cfg = {"workload": workload_text(w), "delta": delta, "merge_prm": args.merge, "setup_s": round(t_setup, 1)}
    for k, v in rec.items():
        if k not in ("seconds", "tokens_per_s", "probe_target_gate_up"):
            cfg[k] = v
    line = {
        "metric": "generated tokens/s (1 GPU) per delta", "value": rec["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": steps_timed, "warmup": 0 if args.until_enomem else args.warmup, "ms_per_step": rec["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.draft.dtype, "data": "synthetic",
        "config": cfg, "roofline": roof,
    }
    if args.sd_k:
        cfg["sd_k"] = args.sd_k
    s.close()
    del s
    torch.cuda.empty_cache()

    if not args.no_extras and not args.until_enomem:
        extras = {}
        # configuration 2 (batch 64, ragged prompts): every delta of its sweep, prompt prefill + a few steps each
        progress("main record done; configuration 2, every delta")
        w2 = workload("cfg2")
        s2 = Session(w2)
        per_delta = {}
        for d in (0.0, 0.5, 0.7, 0.9, 1.01):
            R.rsd_set_criterion(s2.ctx, d)
            per_delta[str(d)] = slim(run_steps(R, s2, w2, 3, 0, probes=(d == 0.7)))
            progress(f"configuration 2, delta {d} done")
        s2.close()
        del s2
        torch.cuda.empty_cache()
        extras["cfg2_per_delta"] = {"workload": workload_text(w2), "steps_timed": 3,
                                    "note": "each delta: prompts set, then 3 reasoning steps, the first of which holds the prompt prefills",
                                    "delta": per_delta}
        # configuration 1 (batch 1, top-p sampling): one whole pass
        progress("configuration 1")
        w1 = workload("cfg1")
        s1 = Session(w1)
        extras["cfg1"] = dict(slim(run_steps(R, s1, w1, w1.max_steps, 2, probes=True, probe_stride=4)), workload=workload_text(w1),
                              delta=w1.delta)
        s1.close()
        del s1
        torch.cuda.empty_cache()
        # configuration 4 (batch 256, 1024-token prompts, 200 GB of KV pools): prompt prefill + 2 steps per delta
        progress("configuration 4")
        w4 = workload("cfg4")
        s4 = Session(w4, kv_pool_bytes=(int(50e9), int(100e9), int(50e9)))
        per_delta4 = {}
        for d in w4.deltas:
            R.rsd_set_criterion(s4.ctx, d)
            per_delta4[str(d)] = slim(run_steps(R, s4, w4, 2, 0, probes=False))
            progress(f"configuration 4, delta {d} done")
        # the decode attention kernel alone on the same caches, every sequence at a context of 4096 tokens (the
        # middle of this configuration's range): one layer launch reads sum(context) x 2 x kv heads x head dim x 2 B
        import numpy as np
        attn4 = {}
        ctx4 = np.full(w4.batch, min(4096, w4.max_ctx), np.int32)
        for which, name in ((0, "draft"), (1, "target")):
            try:
                ms = R.rsd_probe_attention(s4.ctx, which, ctx4, 56)
            except R.RsdError as e:
                attn4[name] = {"error": str(e)}
                continue
            by = int(ctx4.sum()) * 2 * w4.shapes[which].kv_dim * 2
            us = ms / 56 * 1e3
            attn4[name] = {"context": int(ctx4[0]), "bytes_per_launch": by, "avg_launch_us": round(us, 2),
                           "GBs": round(by / us / 1e3, 1), "frac_of_hbm_peak": round(by / us / 1e3 / HBM_PEAK_GBS, 4)}
        s4.close()
        del s4
        torch.cuda.empty_cache()
        extras["cfg4_per_delta"] = {"workload": workload_text(w4), "steps_timed": 2, "kv_pools_GB": [50, 100, 50],
                                    "note": "each delta: prompts set, then 2 reasoning steps (contexts <= 1280); the run to the "
                                            "pool's end is a separate invocation (--workload cfg4 --until-enomem)",
                                    "delta": per_delta4, "decode_attention_kernel": attn4}
        # process Best-of-N (the paper's comparison procedure on the same kernels): the 1.5B base model and reward
        # model of configuration 2, 16 sequences x 4 candidates, the paper's sampling setting for it
        progress("process Best-of-N")
        from paper_2501_19324_amd.harness import BonSession
        wb = replace(workload("cfg2", batch=16), temperature=0.7, top_p=0.8)
        sb = BonSession(wb, 4)
        R.rsd_bon_generate(sb.ctx, max_steps=1, want_tokens=False)           # warm-up: first-use costs
        sb.reset()
        torch.cuda.synchronize()
        tb = time.perf_counter()
        gb = R.rsd_bon_generate(sb.ctx, max_steps=4, want_tokens=False)
        torch.cuda.synchronize()
        tb = time.perf_counter() - tb
        extras["process_best_of_n"] = {"workload": f"{wb.batch} sequences x 4 candidates, draft {wb.draft.n_layers}L-d{wb.draft.d_model} as base model, "
                                                   f"PRM {wb.prm.n_layers}L-d{wb.prm.d_model}, prompts {wb.prompt_len_min}-{wb.prompt_len_max}, "
                                                   f"T={wb.temperature}, top_p={wb.top_p}, prompts set then 4 steps x <= {wb.step_cap} tokens",
                                       "committed_tokens_per_s": round(gb["n_committed"] / tb, 1),
                                       "candidate_tokens_per_s": round(gb["n_draft"] / tb, 1), "seconds": round(tb, 2),
                                       "pages": R.rsd_bon_stats(sb.ctx)}
        sb.close()
        del sb
        torch.cuda.empty_cache()
        line["config"]["other_configs"] = extras
    if not args.no_cpu_baseline:
        progress("GPU records done; timing the CPU checker on its sample (about half a minute)")
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
