"""GPU parity of process Best-of-N (Section 3, "Baselines"): the HIP path, with candidates that
share the committed context's cache pages, against the CPU checker, which evaluates every candidate
on the whole prefix with no sharing at all."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import BonSession
    return dict(R=R, BonSession=BonSession, torch=torch)


def check_pages(R, s, shared_allowed=False):
    """Between steps no page has two owners (sharing exists only inside a step), and used + free = pool."""
    for mdl in (0, 2):
        pg = R.rsd_export_pages(s.ctx, mdl)
        used = pg["block_table"][pg["block_table"] >= 0]
        assert len(set(used.tolist())) == used.size
        assert used.size + pg["free_pages"] == pg["pool_pages"]


@pytest.mark.parametrize("n_cand,sampler", [(1, "greedy"), (3, "sampled"), (4, "sampled")])
def test_tiny_free_running(gpu, tiny, n_cand, sampler):
    """fp32 tiny configuration, free-running: every candidate's tokens, every reward (1e-4), the choice,
    the committed tokens, cache offsets and page counts, step by step."""
    from dataclasses import replace
    from oracle import rsd_oracle as O
    R = gpu["R"]
    w = tiny["w"]
    if sampler == "sampled":
        w = replace(w, temperature=0.7, top_p=0.8, sep_logit_bias=3.5)
    else:
        w = replace(w, sep_logit_bias=0.6)
    s = gpu["BonSession"](w, n_cand)
    d, _, p = tiny["models"]
    P = O.Params(delta=0.0, sep_id=w.sep_id, step_cap=w.step_cap, max_steps=w.max_steps, max_ctx=w.max_ctx, eos_id=w.eos_id,
                 temperature=float(np.float32(w.temperature)), top_p=float(np.float32(w.top_p)),
                 sep_logit_bias=float(np.float32(w.sep_logit_bias)))
    refs = [O.generate_sequence_bon(d, p, s.tokens_host[b, :s.prompt_len[b]], s.u_host[b * n_cand:(b + 1) * n_cand], P, n_cand)
            for b in range(w.batch)]
    chosen = []
    for i in range(w.max_steps):
        g = R.rsd_bon_step(s.ctx)
        for b in range(w.batch):
            r = refs[b]["records"][i]
            for n in range(n_cand):
                assert list(g["cand_tokens"][b, n, :g["cand_len"][b, n]]) == r["candidates"][n], (b, i, n)
                assert abs(float(g["cand_reward"][b, n]) - r["rewards"][n]) < 1e-4
            r32 = np.sort(np.float32(r["rewards"]))
            if n_cand == 1 or r32[-1] - r32[-2] > 2e-4:            # the maximum is clear of the tolerance
                assert g["chosen"][b] == g["own_choice"][b] == r["chosen"], (b, i, g["cand_reward"][b], r["rewards"])
            assert g["ctx_len"][b] == r["ctx_len"] and g["finished"][b] == r["finished"]
            assert list(g["kv_len"][:, b]) == [r["kv_len"][0], r["kv_len"][2]]
            assert list(g["n_pages"][:, b]) == [r["n_pages"][0], r["n_pages"][2]]
            chosen.append(int(g["chosen"][b]))
        check_pages(R, s)
    if n_cand > 1:
        assert len(set(chosen)) > 1
    st = R.rsd_bon_stats(s.ctx)
    if n_cand > 1:
        assert st["pages_shared"] > 0 and st["pages_copied"] > 0
    s.reset()
    out = R.rsd_bon_generate(s.ctx)
    for b in range(w.batch):
        assert list(out["tokens"][b, :out["ctx_len"][b]]) == refs[b]["tokens"]
        assert out["finished"][b] == refs[b]["finished"]
    assert out["n_committed"] == sum(len(r["tokens"]) - r["prompt_len"] for r in refs)
    s.close()


def test_small_pool_needs_the_sharing(gpu, tiny):
    """A pool that could not hold a private copy of the context for every candidate: the run succeeds
    because candidates share the committed pages, and a pool that is too small even so stops with
    RSD_ENOMEM and leaves the sequences as they were."""
    from dataclasses import replace
    R = gpu["R"]
    w = replace(tiny["w"], temperature=0.7, top_p=0.8, sep_logit_bias=3.5)
    n = 4
    kvb = w.draft.kv_bytes_per_token * 16                # bytes of one page, all layers (draft and reward model alike)
    # per sequence: 4 pages hold the longest context; per candidate: 2 pages for its step + 1 copied page
    pages = w.batch * 6 + w.batch * n * 3
    assert pages < w.batch * n * (w.max_ctx // 16)
    s = gpu["BonSession"](w, n, kv_pool_bytes=(pages * kvb, 0, pages * kvb))
    ref = gpu["BonSession"](w, n)
    a, b = R.rsd_bon_generate(s.ctx), R.rsd_bon_generate(ref.ctx)
    assert np.array_equal(a["tokens"], b["tokens"]) and np.array_equal(a["ctx_len"], b["ctx_len"])
    check_pages(R, s)
    s.close(); ref.close()
    tight = gpu["BonSession"](w, n, kv_pool_bytes=(10 * kvb, 0, 10 * kvb))
    with pytest.raises(R.RsdError) as e:
        R.rsd_bon_generate(tight.ctx)
    assert e.value.code == R.RSD_ENOMEM
    st = R.rsd_export_state(tight.ctx, want_tokens=False)
    check_pages(R, tight)
    assert (st["ctx_len"].reshape(w.batch, n)[:, 0] >= tight.prompt_len).all()
    tight.close()


def test_bf16_teacher_forced(gpu):
    """bf16 models at the 1.5B widths (2 layers, vocabulary 4096), 3 sequences x 4 candidates, under
    the teacher (candidate tokens and the choice forced to the checker's): rewards within 2e-2; the
    path's own choice equal to the checker's wherever the two best rewards are more than 1e-3 apart
    (the band the RSD gate's decisions are excused in); cache offsets and page counts exact."""
    import torch
    from oracle import rsd_oracle as O
    from rsd_inputs import workload, model_weights_np
    R = gpu["R"]
    TOL = 2e-2
    n = 4
    w = workload("cfg1", n_layers=2, vocab=4096, batch=3, prompt_len_min=20, prompt_len_max=70, step_cap=8, max_steps=3,
                 temperature=0.0, top_p=1.0, sep_logit_bias=2.3)
    # greedy candidates would all be equal: sample them
    from dataclasses import replace
    w = replace(w, temperature=0.7, top_p=0.8)
    d = O.OracleModel(w.draft, model_weights_np(w.seed, 0, w.draft, threads=8))
    p = O.OracleModel(w.prm, model_weights_np(w.seed, 2, w.prm, threads=8))
    s = gpu["BonSession"](w, n)
    P = O.Params(delta=0.0, sep_id=w.sep_id, step_cap=w.step_cap, max_steps=w.max_steps, max_ctx=w.max_ctx,
                 temperature=float(np.float32(w.temperature)), top_p=float(np.float32(w.top_p)),
                 sep_logit_bias=float(np.float32(w.sep_logit_bias)), kv_dtype="bf16")
    refs = [O.generate_sequence_bon(d, p, s.tokens_host[b, :s.prompt_len[b]], s.u_host[b * n:(b + 1) * n], P, n)
            for b in range(w.batch)]
    fd = np.full((w.batch * n, w.max_steps, w.step_cap), -1, np.int32)
    fc = np.full((w.batch, w.max_steps), -1, np.int32)
    for b, ref in enumerate(refs):
        for r in ref["records"]:
            fc[b, r["step"]] = r["chosen"]
            for k, cand in enumerate(r["candidates"]):
                fd[b * n + k, r["step"], :len(cand)] = cand
    fd_d, fc_d = torch.from_numpy(fd).cuda(), torch.from_numpy(fc).cuda()
    R.rsd_set_teacher(s.ctx, fd_d, None, fc_d)
    s.reset()
    worst, n_choice, n_clear = 0.0, 0, 0
    for i in range(w.max_steps):
        g = R.rsd_bon_step(s.ctx)
        for b in range(w.batch):
            r = refs[b]["records"][i]
            for k in range(n):
                assert list(g["cand_tokens"][b, k, :g["cand_len"][b, k]]) == r["candidates"][k]
                err = abs(float(g["cand_reward"][b, k]) - r["rewards"][k])
                worst = max(worst, err)
                assert err < TOL, (b, i, k, err)
            r_sorted = np.sort(np.asarray(r["rewards"]))
            n_choice += 1
            if r_sorted[-1] - r_sorted[-2] > 1e-3:
                n_clear += 1
                assert g["own_choice"][b] == r["chosen"], (b, i, g["cand_reward"][b], r["rewards"])
            assert g["chosen"][b] == r["chosen"] and g["ctx_len"][b] == r["ctx_len"]
            assert list(g["kv_len"][:, b]) == [r["kv_len"][0], r["kv_len"][2]]
            assert list(g["n_pages"][:, b]) == [r["n_pages"][0], r["n_pages"][2]]
        check_pages(R, s)
    print(f"Best-of-{n} bf16: max reward error {worst:.2e}; choices compared {n_clear} of {n_choice}")
    assert n_clear >= n_choice // 2
    R.rsd_set_teacher(s.ctx, None, None, None)
    s.close()
