"""GPU parity, tiny fp32 configuration: the HIP path against the CPU checker on
the same seeded inputs, free-running (tokens, decisions, KV offsets exact;
logits and rewards within 1e-4)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 1e-4          # logits and rewards, fp32 tiny configuration


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session
    return dict(R=R, Session=Session, torch=torch)


def oracle_params(O, w, **kw):
    base = dict(delta=w.delta, sep_id=w.sep_id, step_cap=w.step_cap, max_steps=w.max_steps, max_ctx=w.max_ctx,
                eos_id=w.eos_id, temperature=float(np.float32(w.temperature)), top_p=float(np.float32(w.top_p)),
                sep_logit_bias=float(np.float32(w.sep_logit_bias)), omega_kind=w.omega_kind,
                omega_a=float(np.float32(w.omega_a)))
    base.update(kw)
    return O.Params(**base)


@pytest.mark.parametrize("chunk", [1, 5, 64])
def test_forward_logits_and_rewards(gpu, tiny, chunk):
    """Teacher-forced logits of draft and target and rewards of the reward
    model at every position: single-token decode kernels (chunk 1), chunked
    prefill with ragged pieces (chunk 5) and one-shot prefill (chunk 64)."""
    from oracle import rsd_oracle as O
    R = gpu["R"]
    w = tiny["w"]
    s = gpu["Session"](w)
    rng = np.random.default_rng(5)
    T = 40
    lens = np.array([40, 17, 33, 1], dtype=np.int32)
    toks = rng.integers(0, w.draft.vocab, size=(w.batch, T)).astype(np.int32)
    for which in (0, 1, 2):
        out = R.rsd_forward(s.ctx, which, toks, lens, chunk).cpu().numpy()
        m = tiny["models"][which]
        for b in range(w.batch):
            y = O.forward_full(m, [int(t) for t in toks[b, :lens[b]]])
            if which == 2:
                ref = np.array([O.reward(m, y[i]) for i in range(lens[b])])
                got = out[b, :lens[b]]
            else:
                ref = O.lm_logits(m, y)
                got = out[b, :lens[b], :]
            err = np.max(np.abs(got - ref))
            assert err < TOL, (which, b, chunk, err)
            assert np.all(np.isnan(out[b, lens[b]:]))
    s.close()


def test_sampler_alone(gpu):
    """The sampler kernel on given logits against the checker's definition:
    arg max with ties, and nucleus draws over several temperatures / top_p."""
    from oracle import rsd_oracle as O
    R, torch = gpu["R"], gpu["torch"]
    from rsd_inputs import workload
    s = gpu["Session"](workload("cfg0"))
    rng = np.random.default_rng(9)
    n, V = 64, 1024
    lg = (rng.normal(size=(n, V)) * 0.8).astype(np.float32)
    lg[3, 100] = lg[3, 900] = lg[3].max() + 1.0          # tie: lowest id wins
    lg[4, :] = 0.25                                        # all equal
    u = rng.random(n).astype(np.float32)
    lg_d, u_d = torch.from_numpy(lg).cuda(), torch.from_numpy(u).cuda()
    got = R.rsd_sample(s.ctx, lg_d, None, 0.0, 1.0).cpu().numpy()
    assert list(got) == [O.sample(lg[i], 0.0, 0.0, 1.0) for i in range(n)]
    assert got[3] == 100 and got[4] == 0
    for T, top_p in ((0.7, 0.95), (1.0, 1.0), (0.7, 0.5), (1.3, 0.05), (0.7, 0.0)):
        got = R.rsd_sample(s.ctx, lg_d, u_d, T, top_p).cpu().numpy()
        bad = 0
        for i in range(n):
            ref = O.sample(lg[i], float(u[i]), float(np.float32(T)), float(np.float32(top_p)))
            bad += int(got[i] != ref)
        assert bad == 0, (T, top_p, bad)
    # larger vocabulary with a ragged tail
    V2 = 151936
    lg2 = (rng.normal(size=(6, V2)) * 0.8).astype(np.float32)
    u2 = rng.random(6).astype(np.float32)
    got = R.rsd_sample(s.ctx, torch.from_numpy(lg2).cuda(), torch.from_numpy(u2).cuda(), 0.7, 0.95).cpu().numpy()
    for i in range(6):
        ref = O.sample(lg2[i], float(u2[i]), float(np.float32(0.7)), float(np.float32(0.95)))
        assert got[i] == ref, (i, got[i], ref)
    s.close()


def run_and_compare(gpu, tiny, w, n_steps=None, models=None, merge=0):
    from oracle import rsd_oracle as O
    R = gpu["R"]
    s = gpu["Session"](w, merge_prm=merge)
    P = oracle_params(O, w, merge=("none", "draft", "target")[merge])
    n_steps = n_steps or w.max_steps
    models = models or tiny["models"]
    refs = [O.generate_sequence(*models, s.tokens_host[b, :s.prompt_len[b]], s.u_host["U_DRAFT"][b],
                                s.u_host["U_TARGET"][b], s.u_host["U_GATE"][b], P) for b in range(w.batch)]
    n_acc = n_rej = 0
    for i in range(n_steps):
        if all(len(r["records"]) <= i for r in refs):
            break
        g = R.rsd_step(s.ctx)
        st = R.rsd_export_state(s.ctx)
        for b in range(w.batch):
            if len(refs[b]["records"]) <= i:
                assert g["draft_len"][b] == 0 and g["final_len"][b] == 0
                continue
            r = refs[b]["records"][i]
            assert list(g["draft_tokens"][b, :g["draft_len"][b]]) == r["draft_tokens"], (b, i)
            assert abs(float(g["reward"][b]) - r["reward"]) < TOL, (b, i)
            assert bool(g["accepted"][b]) == r["accepted"] and g["accepted"][b] == g["own_accept"][b], (b, i)
            assert list(g["final_tokens"][b, :g["final_len"][b]]) == r["final_tokens"], (b, i)
            assert g["finished"][b] == r["finished"], (b, i)
            assert st["ctx_len"][b] == r["ctx_len"]
            assert list(st["kv_len"][:, b]) == r["kv_len"], (b, i, st["kv_len"][:, b], r["kv_len"])
            assert list(st["n_pages"][:, b]) == r["n_pages"], (b, i)
            n_acc += r["accepted"]
            n_rej += not r["accepted"]
        # page tables: no page owned twice, used + free = pool
        for m in range(3 if merge == 0 else 2):
            pg = R.rsd_export_pages(s.ctx, m)
            used = pg["block_table"][pg["block_table"] >= 0]
            assert len(set(used.tolist())) == used.size
            assert used.size + pg["free_pages"] == pg["pool_pages"]
            assert np.array_equal((pg["block_table"] >= 0).sum(1), st["n_pages"][m])
    st = R.rsd_export_state(s.ctx)
    for b in range(w.batch):
        n = st["ctx_len"][b]
        assert list(st["tokens"][b, :n]) == refs[b]["tokens"][:n]
    # the target's stages serve the rejected sequences only: their iterations run over packed rows, never
    # fewer rows than sequences in them and (once a step was accepted somewhere) fewer than the batch
    it = R.rsd_iter_stats(s.ctx, R.RSD_TARGET)
    assert it["seq_iterations"] <= it["row_iterations"] <= w.batch * it["iterations"]
    if n_acc >= 2 and n_rej >= 2 and merge == 0 and 4 <= w.batch <= 8 and it["iterations"]:
        assert it["row_iterations"] < w.batch * it["iterations"], it
    s.close()
    return n_acc, n_rej


def test_config0_free_running(gpu, tiny):
    """Config 0 as written: greedy, delta 0.5, 4 steps of <= 16 tokens."""
    run_and_compare(gpu, tiny, tiny["w"])


def test_config0_ragged_steps_greedy(gpu, tiny):
    from rsd_inputs import workload
    w = workload("cfg0", sep_logit_bias=0.6, deltas=(0.55,))
    n_acc, n_rej = run_and_compare(gpu, tiny, w)
    assert n_acc >= 2 and n_rej >= 2


def test_config0_ragged_steps_sampled(gpu, tiny):
    from rsd_inputs import workload
    w = workload("cfg0", sep_logit_bias=3.5, deltas=(0.55,), temperature=0.7, top_p=0.95)
    n_acc, n_rej = run_and_compare(gpu, tiny, w)
    assert n_acc >= 2 and n_rej >= 2


def test_config0_eos_and_context_limit(gpu, tiny):
    from rsd_inputs import workload
    w = workload("cfg0", sep_logit_bias=3.5, deltas=(0.55,), temperature=0.7, top_p=0.95, eos_id=517, max_steps=5)
    run_and_compare(gpu, tiny, w)


@pytest.mark.parametrize("delta,which", [(0.0, 0), (1.01, 1)])
def test_gate_fixed_points_on_gpu(gpu, tiny, delta, which):
    """delta <= 0 is draft-only decoding, delta > 1 target-only, token for token."""
    from oracle import rsd_oracle as O
    from rsd_inputs import workload
    R = gpu["R"]
    w = workload("cfg0", deltas=(delta,), sep_logit_bias=0.6)
    s = gpu["Session"](w)
    out = R.rsd_generate(s.ctx)
    P = oracle_params(O, w)
    for b in range(w.batch):
        n = out["ctx_len"][b] - s.prompt_len[b]
        ref = O.decode_plain(tiny["models"][which], s.tokens_host[b, :s.prompt_len[b]],
                             s.u_host["U_DRAFT" if which == 0 else "U_TARGET"][b], P, int(n))
        assert list(out["tokens"][b, s.prompt_len[b]:out["ctx_len"][b]]) == ref
    assert (out["n_reject"] == 0) if which == 0 else (out["n_accept"] == 0)
    st = R.rsd_export_state(s.ctx)
    if which == 0:
        assert np.all(st["kv_len"][1] == 0)
    s.close()


def test_teacher_forcing_and_generate_twice(gpu, tiny):
    """Under a teacher the appended tokens and decisions are the forced ones
    while the path's own choices are still reported; two runs of the same
    inputs give identical results."""
    from rsd_inputs import workload
    R, torch = gpu["R"], gpu["torch"]
    w = workload("cfg0", sep_logit_bias=0.6, deltas=(0.55,))
    s = gpu["Session"](w)
    a = R.rsd_generate(s.ctx)
    s.reset()
    b = R.rsd_generate(s.ctx)
    assert np.array_equal(a["tokens"], b["tokens"]) and np.array_equal(a["ctx_len"], b["ctx_len"])
    own_d, own_t = R.rsd_export_sampled(s.ctx)
    # force the same trajectory but flip every decision of step 0 to "accept"
    fd = torch.from_numpy(own_d).cuda()
    ft = torch.from_numpy(own_t).cuda()
    fa = torch.full((w.batch, w.max_steps), -1, dtype=torch.int32, device="cuda")
    fa[:, 0] = 1
    R.rsd_set_teacher(s.ctx, fd, ft, fa)
    s.reset()
    g = R.rsd_step(s.ctx)
    assert np.all(g["accepted"] == 1)
    assert np.array_equal(g["final_tokens"], g["draft_tokens"])
    R.rsd_set_teacher(s.ctx, None, None, None)
    s.close()


def test_pool_exhaustion_leaves_state_unchanged(gpu, tiny):
    from rsd_inputs import workload
    R = gpu["R"]
    w = workload("cfg0")
    page_bytes = 2 * w.draft.n_kv_heads * 16 * w.draft.head_dim * 4 * w.draft.n_layers
    s = gpu["Session"](w, kv_pool_bytes=(page_bytes * 13, 0, 0))       # 4 sequences x 3 pages + 1
    R.rsd_step(s.ctx)           # 32 + 16 tokens: 3 pages each, fits
    before = R.rsd_export_state(s.ctx)
    with pytest.raises(R.RsdError) as e:
        R.rsd_step(s.ctx)       # would need a fourth page for every sequence
    assert e.value.code == R.RSD_ENOMEM
    after = R.rsd_export_state(s.ctx)
    for k in ("ctx_len", "kv_len", "n_pages", "tokens"):
        assert np.array_equal(before[k], after[k])
    s.close()


def test_bad_arguments_are_rejected(gpu, tiny):
    from rsd_inputs import workload
    from dataclasses import replace
    R = gpu["R"]
    w = workload("cfg0")
    s = gpu["Session"](w)
    with pytest.raises(R.RsdError) as e:
        R.rsd_init([replace(w.draft, n_heads=3), w.target, w.prm], s.weights, batch=4, delta=0.5, sep_id=1023,
                   step_cap=16, max_steps=4, max_ctx=96)
    assert e.value.code == R.RSD_EINVAL
    with pytest.raises(R.RsdError):
        R.rsd_init(w.shapes, s.weights, batch=4, delta=0.5, sep_id=5000, step_cap=16, max_steps=4, max_ctx=96)
    with pytest.raises(R.RsdError):
        R.rsd_set_prompts(s.ctx, s.tokens, np.array([32, 32, 0, 32], np.int32))
    out = R.rsd_generate(s.ctx)
    with pytest.raises(R.RsdError) as e:
        R.rsd_step(s.ctx)
    assert e.value.code == R.RSD_ESTATE and out["steps_run"] == 4
    s.close()


@pytest.mark.parametrize("kind,a", [(1, 0.6), (2, 0.0), (3, 0.0), (4, 8.0)])
def test_general_weightings_on_gpu(gpu, tiny, kind, a):
    """Table 1's other weighting functions (constant, clipped, r / (1 + r), logistic) through
    Algorithm 2's uniform draw: rewards, decisions, tokens and offsets against the checker."""
    from rsd_inputs import workload
    w = workload("cfg0", omega_kind=kind, omega_a=a, sep_logit_bias=0.6, deltas=(0.55,), max_steps=6)
    n_acc, n_rej = run_and_compare(gpu, tiny, w)
    assert n_acc >= 1 and n_rej >= 1


@pytest.mark.parametrize("batch,plen,cap", [(1, 1, 1), (2, 1, 3), (5, 17, 1)])
def test_smallest_inputs(gpu, tiny, batch, plen, cap):
    """One-token prompts, one-token steps, a single sequence."""
    from rsd_inputs import workload
    w = workload("cfg0", batch=batch, prompt_len_min=plen, prompt_len_max=plen, step_cap=cap, max_steps=5,
                 sep_logit_bias=0.6, deltas=(0.5,))
    run_and_compare(gpu, tiny, w)


@pytest.mark.parametrize("kind,a", [(0, 0.0), (3, 0.0)])
def test_one_step_law_is_the_mixture_on_gpu(gpu, kind, a):
    """Proposition 1 through the HIP path: with one-token steps the committed first token of a
    sequence is distributed as omega_r P_m + nu P_M.  4096 sequences share one prompt and differ
    only in their uniforms; P_m, P_M and the rewards come from the checker.  Vocabulary of 8 ids
    so that 4096 draws settle every cell."""
    from oracle import rsd_oracle as O
    from rsd_inputs import workload, model_weights_np
    R, torch = gpu["R"], gpu["torch"]
    n = 4096
    w0 = workload("cfg0", vocab=8, batch=n, prompt_len_min=6, prompt_len_max=6, step_cap=1, max_steps=1,
                  temperature=1.0, top_p=1.0, sep_logit_bias=0.0, omega_kind=kind, omega_a=a)
    models = [O.OracleModel(s, model_weights_np(w0.seed, i, s)) for i, s in enumerate(w0.shapes)]
    from rsd_inputs import prompt_tokens
    prompt = [int(t) for t in prompt_tokens(w0)[0, :6]]
    p_m = O.softmax(O.lm_logits(models[0], O.forward_full(models[0], prompt)[-1]))
    p_M = O.softmax(O.lm_logits(models[1], O.forward_full(models[1], prompt)[-1]))
    rew = np.array([O.reward(models[2], O.forward_full(models[2], prompt + [i])[-1]) for i in range(8)])
    delta = float(np.float32(np.median(rew)))
    wts = np.array([O.omega(x, kind, delta, a) for x in rew])
    assert 0 < wts.sum() < 8
    expect, nu = O.mixture_distribution(p_m, p_M, wts)

    from dataclasses import replace
    w = replace(w0, deltas=(delta,))
    s = gpu["Session"](w)
    s.tokens_host[:, :6] = np.array(prompt, np.int32)[None, :]
    s.tokens = torch.from_numpy(s.tokens_host).cuda()
    s.reset()
    g = R.rsd_step(s.ctx)
    assert np.all(g["final_len"] == 1)
    counts = np.bincount(g["final_tokens"][:, 0], minlength=8).astype(np.float64)
    n_rej = int(np.sum(g["accepted"] == 0))
    chi2 = np.sum((counts - n * expect) ** 2 / (n * expect))
    assert chi2 < 35.0, (chi2, counts, n * expect)                 # 7 dof: P(chi2 > 35) ~ 1e-5
    assert abs(n_rej / n - nu) < 5 * np.sqrt(nu * (1 - nu) / n), (n_rej / n, nu)
    s.close()


@pytest.mark.parametrize("merge", [1, 2])
def test_merged_reward_head_on_gpu(gpu, tiny, merge):
    """Appendix "Model Merge": the reward head on the draft's (1) or the target's (2) trunk, no third
    model or cache.  Free-running against the checker: tokens, rewards, decisions, offsets, pages."""
    from dataclasses import replace
    from oracle import rsd_oracle as O
    from rsd_inputs import workload, model_weights_np
    w = workload("cfg0", sep_logit_bias=0.6, deltas=(0.5,), max_steps=6)
    policy = w.draft if merge == 1 else w.target
    w = replace(w, prm=replace(policy, head_kind="reward"))
    d, t, _ = tiny["models"]
    head = model_weights_np(w.seed, 2, w.prm)
    trunk = (d if merge == 1 else t)._w
    pm = O.OracleModel(w.prm, {**{k: v for k, v in trunk.items() if k != "lm_head"}, "w_r": head["w_r"], "b_r": head["b_r"]})
    n_acc, n_rej = run_and_compare(gpu, tiny, w, models=(d, t, pm), merge=merge)
    assert n_acc >= 2 and n_rej >= 2


def test_table_check_accepts_what_is_owned_and_names_what_is_not(gpu, tiny):
    """rsd_check_rows against the state after one reasoning step: rows inside the pages their sequences own
    pass; a position behind the owned pages, a sequence outside the batch and a position outside the context
    limit are each refused with RSD_ESTATE and named, by a kernel that only reads what it has checked."""
    R = gpu["R"]
    w = tiny["w"]
    s = gpu["Session"](w)
    R.rsd_step(s.ctx)
    st = R.rsd_export_state(s.ctx, want_tokens=False)
    for m in range(3):
        owned = st["n_pages"][m] * w.page_tokens
        has = np.flatnonzero(owned > 0)          # (the target owns nothing for a sequence it has not been asked about)
        if not has.size:
            with pytest.raises(R.RsdError) as e:
                R.rsd_check_rows(s.ctx, m, np.array([0]), np.array([0]))
            assert e.value.code == R.RSD_ESTATE and "beyond the pages" in str(e.value)
            continue
        R.rsd_check_rows(s.ctx, m, np.repeat(has, 2), np.stack([np.zeros(has.size, np.int64), owned[has] - 1], 1).reshape(-1))
        for bad_seq, bad_pos, what in ((0, int(owned[0]), "beyond the pages"), (w.batch, 0, "outside the batch"),
                                       (-1, 0, "outside the batch"), (1, w.max_ctx, "outside the context limit"),
                                       (1, -1, "outside the context limit")):
            if what == "beyond the pages" and bad_pos >= w.max_ctx:
                continue
            with pytest.raises(R.RsdError) as e:
                R.rsd_check_rows(s.ctx, m, np.array([int(has[0]), bad_seq]), np.array([0, bad_pos]))
            assert e.value.code == R.RSD_ESTATE and what in str(e.value) and "row 1" in str(e.value), str(e.value)
    R.rsd_step(s.ctx)            # the context is still usable
    s.close()


def test_checked_build_runs_the_tiny_configuration(gpu, tiny):
    """The library built with the table check before every pass and every single-token iteration
    (librsd_debug.so): same tokens, decisions, rewards and offsets as the checker, no graph replays, and a
    pool that runs out is still a clean RSD_ENOMEM (the check sees the state the failed call restored)."""
    import os
    from rsd_inputs import workload
    R = gpu["R"]
    path = os.path.join(os.path.dirname(R.LIB_PATH), "librsd_debug.so")
    release = R.load_library()
    try:
        R.load_library(path)
        assert R.rsd_debug_build()
        w = workload("cfg0", sep_logit_bias=0.6, deltas=(0.55,))
        n_acc, n_rej = run_and_compare(gpu, tiny, w)
        assert n_acc >= 2 and n_rej >= 2
        s = gpu["Session"](w)
        R.rsd_generate(s.ctx)
        ds = R.rsd_decode_stats(s.ctx)
        assert ds["eager_iters"] > 0 and ds["graph_replays"] == 0
        s.close()
        page_bytes = 2 * w.draft.n_kv_heads * 16 * w.draft.head_dim * 4 * w.draft.n_layers
        small = gpu["Session"](w, kv_pool_bytes=(page_bytes * 13, 0, 0))       # 4 sequences x 3 pages + 1
        R.rsd_step(small.ctx)
        with pytest.raises(R.RsdError) as e:
            for _ in range(w.max_steps):
                R.rsd_step(small.ctx)
        assert e.value.code == R.RSD_ENOMEM
        small.close()
    finally:
        R._lib = release
    assert not R.rsd_debug_build()
