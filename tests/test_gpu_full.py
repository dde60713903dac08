"""GPU checks at full depth and full width (bf16, 28-layer 1.5B draft / 7B target /
1.5B reward model, vocabulary 151936), in the launch configurations bench.py times:
configuration 1 (batch 1), seeded subsets of configurations 2 (batch 64, ragged
prompts), 4 (batch 256, 1024-token prompts) and 3 (batch 16, 72B target resident, 7B
reward model), and two whole reasoning steps of configuration 3 checked by properties.

The fp64 CPU checker can evaluate all three full-depth models on a prompt (the 7B
target is about 60 GB as fp64), so next-token logits and rewards are compared with
it directly; whole free runs at this size would take the checker hours and are
covered by properties that hold at any size."""
import gc

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 2e-2


@pytest.fixture(scope="module")
def full():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from rsd_inputs import workload
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session
    w = workload("cfg1")
    s = Session(w)
    yield dict(R=R, s=s, w=w, torch=torch)
    s.close()


@pytest.fixture(scope="module")
def checker_models():
    """Full-depth checker models of a configuration (its own seed), built on first use; one configuration
    is kept at a time."""
    from oracle import rsd_oracle as O
    from rsd_inputs import model_weights_np, workload
    cache = {}

    def get(name, which):
        if (name, which) not in cache:
            for k in [k for k in cache if k[0] != name]:
                del cache[k]
            gc.collect()
            w = workload(name)
            cache[(name, which)] = O.OracleModel(w.shapes[which], model_weights_np(w.seed, which, w.shapes[which], threads=16))
        return cache[(name, which)]
    get.drop = lambda name, which: (cache.pop((name, which), None), gc.collect())
    return get


# Against the checker that keeps cache entries exact the error is dominated by the bf16 storage of keys and
# values itself (the two checkers differ by as much): 2.3e-2 on the 1.5B logits, 1.0e-1 on the 7B logits,
# 9e-4 on rewards when measured.  Stated bounds for the record, not the parity tolerance:
EXACT_KV_BOUND = {0: 1e-1, 1: 3e-1, 2: 5e-3}


@pytest.mark.parametrize("which", [0, 2, 1])
def test_full_depth_prompt_against_checker(full, checker_models, which):
    """Last-position logits of the draft (which = 0) and of the 7B target (1) and the reward of the
    reward model (2) on the 256-token prompt, through the chunked prefill kernels and through 256
    single-token iterations.  Compared with the checker that stores cache entries as bf16 (the
    tolerance of the parity statement) and, for the record, with the checker that keeps them exact."""
    from oracle import rsd_oracle as O
    R, s, w = full["R"], full["s"], full["w"]
    n = int(s.prompt_len[0])
    toks = s.tokens_host[:, :n].copy()
    lens = np.array([n], np.int32)
    m = checker_models("cfg1", which)
    seq = [int(t) for t in toks[0]]
    head = (lambda y: O.lm_logits(m, y)) if which != 2 else (lambda y: np.array(O.reward(m, y)))
    ref = head(O.forward_full(m, seq, "bf16")[-1])
    ref_exact = head(O.forward_full(m, seq, "exact")[-1])
    print(f"model {which}: the two checkers differ by {float(np.max(np.abs(ref - ref_exact))):.2e} (bf16 against exact cache entries)")
    if which == 1:
        checker_models.drop("cfg1", 1)
    for chunk in (n, 1):
        out = R.rsd_forward(s.ctx, which, toks, lens, chunk)
        got = out[0, n - 1].cpu().numpy()
        err = float(np.max(np.abs(got - ref)))
        err_exact = float(np.max(np.abs(got - ref_exact)))
        print(f"model {which} chunk {chunk}: max abs error {err:.2e} (bf16 cache entries in the checker), "
              f"{err_exact:.2e} (exact cache entries in the checker)")
        assert err < (TOL if which != 2 else 1e-3), (which, chunk, err)
        assert err_exact < EXACT_KV_BOUND[which], (which, chunk, err_exact)
    s.reset()


@pytest.mark.parametrize("name,check", [("cfg2", [5, 40]), ("cfg4", [17]), ("cfg3", [3])])
def test_full_depth_batched_subset(checker_models, name, check):
    """Configurations 2, 4 and 3 at their own batch (64 / 256 / 16; configuration 3 with its 72B target
    resident and its 7B reward model scoring), prompts and full-depth models, steps
    truncated to 12 tokens: the sequences in `check` are followed by the checker for two reasoning
    steps under the teacher (draft tokens forced, delta = 0 so that the target, whose full-depth
    checker costs minutes per step, is never needed): draft tokens (the path's own choice may differ
    only at a near-tie), rewards, cache offsets and page counts."""
    import torch
    from oracle import rsd_oracle as O
    from rsd_inputs import workload
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session
    w = workload(name, step_cap=12, max_steps=2, deltas=(0.0,))
    s = Session(w)
    P = O.Params(delta=0.0, sep_id=w.sep_id, step_cap=w.step_cap, max_steps=w.max_steps, max_ctx=w.max_ctx, kv_dtype="bf16")
    md, mp = checker_models(name, 0), checker_models(name, 2)
    # (the target's place is taken by the draft model: with delta = 0 every step is accepted and it is never run)
    refs = {b: O.generate_sequence(md, md, mp, s.tokens_host[b, :s.prompt_len[b]], s.u_host["U_DRAFT"][b],
                                   s.u_host["U_TARGET"][b], s.u_host["U_GATE"][b], P) for b in check}
    fd = np.full((w.batch, w.max_steps, w.step_cap), -1, np.int32)
    for b, ref in refs.items():
        for r in ref["records"]:
            fd[b, r["step"], :len(r["draft_tokens"])] = r["draft_tokens"]
    fd_dev = torch.from_numpy(fd).cuda()
    R.rsd_set_teacher(s.ctx, fd_dev, None, None)
    s.reset()
    worst = 0.0
    for i in range(w.max_steps):
        g = R.rsd_step(s.ctx)
        st = R.rsd_export_state(s.ctx, want_tokens=False)
        assert g["accepted"].all()
        for b in check:
            r = refs[b]["records"][i]
            worst = max(worst, abs(float(g["reward"][b]) - r["reward"]))
            assert abs(float(g["reward"][b]) - r["reward"]) < TOL, (b, i, g["reward"][b], r["reward"])
            assert list(g["final_tokens"][b, :g["final_len"][b]]) == r["final_tokens"]
            assert list(st["kv_len"][:, b]) == r["kv_len"] and list(st["n_pages"][:, b]) == r["n_pages"]
            assert st["ctx_len"][b] == r["ctx_len"]
    own_d, _ = R.rsd_export_sampled(s.ctx)
    n_tok = excused = 0
    for b in check:
        for r in refs[b]["records"]:
            for j, t in enumerate(r["draft_tokens"]):
                n_tok += 1
                if own_d[b, r["step"], j] != t:
                    assert r["draft_margins"][j] < 2 * TOL, (b, r["step"], j, r["draft_margins"][j])
                    excused += 1
    print(f"{name}: {len(check)} sequences followed, {n_tok} draft tokens compared, {excused} excused near-ties, "
          f"max reward error {worst:.2e}")
    for mdl in range(3):
        pg = R.rsd_export_pages(s.ctx, mdl)
        used = pg["block_table"][pg["block_table"] >= 0]
        assert len(set(used.tolist())) == used.size and used.size + pg["free_pages"] == pg["pool_pages"]
    R.rsd_set_teacher(s.ctx, None, None, None)
    s.close()


def test_full_size_steps_properties(full):
    """Three reasoning steps at full size, twice: identical results, offsets and
    page tables consistent with the decisions, rewards inside (0, 1)."""
    R, s, w = full["R"], full["s"], full["w"]
    runs = []
    for _ in range(2):
        s.reset()
        recs, states = [], []
        for _i in range(3):
            recs.append(R.rsd_step(s.ctx))
            states.append(R.rsd_export_state(s.ctx, want_tokens=False))
        runs.append((recs, states, R.rsd_export_state(s.ctx)["tokens"].copy()))
    (ra, sa, ta), (rb, sb, tb) = runs
    assert np.array_equal(ta, tb)
    for x, y in zip(ra, rb):
        for k in x:
            assert np.array_equal(x[k], y[k]), k
    kv_t_prev = 0
    ctx = int(s.prompt_len[0])
    for g, st in zip(ra, sa):
        assert 0.0 < g["reward"][0] < 1.0
        assert g["accepted"][0] == g["own_accept"][0] == int(g["reward"][0] >= np.float32(w.delta))
        assert 1 <= g["draft_len"][0] <= w.step_cap and 1 <= g["final_len"][0] <= w.step_cap
        pre, ctx = ctx, ctx + int(g["final_len"][0])
        kd, kt, kp = (int(v) for v in st["kv_len"][:, 0])
        assert st["ctx_len"][0] == ctx
        if g["accepted"][0]:
            assert (kd, kt, kp) == (ctx - 1, kv_t_prev, ctx)
            assert np.array_equal(g["draft_tokens"], g["final_tokens"])
        else:
            assert (kd, kt, kp) == (pre, ctx - 1, pre)
        assert list(st["n_pages"][:, 0]) == [-(-v // 16) for v in (kd, kt, kp)]
        kv_t_prev = kt
    for mdl in range(3):
        pg = R.rsd_export_pages(s.ctx, mdl)
        used = pg["block_table"][pg["block_table"] >= 0]
        assert len(set(used.tolist())) == used.size and used.size + pg["free_pages"] == pg["pool_pages"]


def test_largest_configuration_steps_properties():
    """Configuration 3 as bench.py times it (batch 16, 1.5B draft, 72B target, 7B reward model, 512-token
    prompts, steps of up to 128 tokens): two reasoning steps, twice.  The 72B target is beyond the checker
    (580 GB in fp64), so what holds at any size is checked for every sequence: identical results on the
    second run, decisions equal to the threshold rule on the exported rewards, the cache-offset and page
    contract of accepted and rejected steps, no page owned twice, and rows of the target's stages packed
    to the rejected sequences."""
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from rsd_inputs import workload
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session
    w = workload("cfg3", max_steps=2)
    s = Session(w)
    runs = []
    for _ in range(2):
        s.reset()
        R.rsd_iter_stats(s.ctx, R.RSD_TARGET, reset=True)
        recs, states = [], []
        for _i in range(w.max_steps):
            recs.append(R.rsd_step(s.ctx))
            states.append(R.rsd_export_state(s.ctx, want_tokens=False))
        runs.append((recs, states, R.rsd_export_state(s.ctx)["tokens"].copy(), R.rsd_iter_stats(s.ctx, R.RSD_TARGET)))
    (ra, sa, ta, ia), (rb, sb, tb, ib) = runs
    assert np.array_equal(ta, tb)
    for x, y in zip(ra, rb):
        for k in x:
            assert np.array_equal(x[k], y[k]), k
    ctx = s.prompt_len.astype(np.int64).copy()
    kv_t_prev = np.zeros(w.batch, np.int64)
    n_rej = 0
    for g, st in zip(ra, sa):
        assert ((g["reward"] > 0.0) & (g["reward"] < 1.0)).all()
        assert np.array_equal(g["accepted"] != 0, g["reward"] >= np.float32(w.delta))
        assert np.array_equal(g["accepted"], g["own_accept"])
        assert ((g["draft_len"] >= 1) & (g["draft_len"] <= w.step_cap) & (g["final_len"] >= 1) & (g["final_len"] <= w.step_cap)).all()
        pre, ctx = ctx, ctx + g["final_len"]
        assert np.array_equal(st["ctx_len"], ctx)
        for b in range(w.batch):
            kd, kt, kp = (int(v) for v in st["kv_len"][:, b])
            if g["accepted"][b]:
                assert (kd, kt, kp) == (ctx[b] - 1, kv_t_prev[b], ctx[b]), b
                assert np.array_equal(g["draft_tokens"][b], g["final_tokens"][b])
            else:
                assert (kd, kt, kp) == (pre[b], ctx[b] - 1, pre[b]), b
                n_rej += 1
            assert list(st["n_pages"][:, b]) == [-(-v // 16) for v in (kd, kt, kp)]
        kv_t_prev = st["kv_len"][1].astype(np.int64)
    assert n_rej > 0, "the target never ran"
    assert ia["iterations"] > 0 and ia["seq_iterations"] <= ia["row_iterations"] <= w.batch * ia["iterations"]
    assert ia == {**ib, "gpu_ms": ia["gpu_ms"]}
    for mdl in range(3):
        pg = R.rsd_export_pages(s.ctx, mdl)
        used = pg["block_table"][pg["block_table"] >= 0]
        assert len(set(used.tolist())) == used.size and used.size + pg["free_pages"] == pg["pool_pages"]
    print(f"configuration 3: {n_rej} of {2 * w.batch} steps regenerated by the 72B target; its iterations ran on "
          f"{ia['row_iterations'] / ia['iterations']:.1f} rows on average for {ia['seq_iterations'] / ia['iterations']:.1f} sequences")
    s.close()
