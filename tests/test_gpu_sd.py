"""GPU parity of the speculative regeneration of rejected steps (Section 5,
"Combine RSD with SD"; greedy, as the paper runs SD): the HIP path against the
CPU checker on the same seeded inputs - committed tokens, the draft's proposals,
rounds / proposals / kept counts and KV offsets exact in the tiny fp32
configuration; under a teacher in bf16."""
from dataclasses import replace

import numpy as np
import pytest

from test_gpu_tiny import gpu, oracle_params, TOL  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def compare_sd(gpu, w, models, sd_k, merge=0, weights=None, min_margin=0.0):
    """min_margin: sequences in which the checker met a top-2 logit gap below it (a near-tie the fp32
    path may resolve the other way) still run but are not compared."""
    from oracle import rsd_oracle as O
    R = gpu["R"]
    s = gpu["Session"](w, merge_prm=merge, sd_k=sd_k, weights=weights)
    P = oracle_params(O, w, merge=("none", "draft", "target")[merge], sd_k=sd_k)
    sampled = w.temperature > 0
    refs = [O.generate_sequence(*models, s.tokens_host[b, :s.prompt_len[b]], s.u_host["U_DRAFT"][b],
                                s.u_host["U_TARGET"][b], s.u_host["U_GATE"][b], P,
                                u_prop=s.u_host["U_PROP"][b] if sampled else None,
                                u_acc=s.u_host["U_ACC"][b] if sampled else None) for b in range(w.batch)]
    tot = dict(rej=0, rounds=0, prop=0, kept=0, skipped=0)
    skip = set()
    for b, ref in enumerate(refs):
        gaps = [x for r in ref["records"] for x in r["draft_margins"] + r["final_margins"] + r["proposal_margins"]]
        if min(gaps) < min_margin:
            skip.add(b)
    tot["skipped"] = len(skip)
    for i in range(w.max_steps):
        if all(len(r["records"]) <= i for r in refs):
            break
        g = R.rsd_step(s.ctx)
        st = R.rsd_export_state(s.ctx)
        for b in range(w.batch):
            if b in skip:
                continue
            if len(refs[b]["records"]) <= i:
                assert g["final_len"][b] == 0
                continue
            r = refs[b]["records"][i]
            assert list(g["draft_tokens"][b, :g["draft_len"][b]]) == r["draft_tokens"], (b, i)
            assert abs(float(g["reward"][b]) - r["reward"]) < TOL, (b, i)
            assert bool(g["accepted"][b]) == r["accepted"], (b, i)
            assert list(g["final_tokens"][b, :g["final_len"][b]]) == r["final_tokens"], (b, i)
            assert g["finished"][b] == r["finished"], (b, i)
            assert st["ctx_len"][b] == r["ctx_len"]
            assert list(st["kv_len"][:, b]) == r["kv_len"], (b, i, st["kv_len"][:, b], r["kv_len"])
            assert list(st["n_pages"][:, b]) == r["n_pages"], (b, i)
            rounds = r["sd_rounds"]
            assert g["sd_rounds"][b] == len(rounds), (b, i, g["sd_rounds"][b], rounds)
            assert g["sd_proposed"][b] == sum(p for p, _ in rounds) and g["sd_kept"][b] == sum(k for _, k in rounds), (b, i, rounds)
            tot["rej"] += not r["accepted"]
            tot["rounds"] += len(rounds); tot["prop"] += sum(p for p, _ in rounds); tot["kept"] += sum(k for _, k in rounds)
    prop, flags = R.rsd_export_proposed(s.ctx, want_flags=True)
    _, own_t = R.rsd_export_sampled(s.ctx)
    for b in range(w.batch):
        if b in skip:
            continue
        want = np.full(prop.shape[1:], -1, np.int32)
        for r in refs[b]["records"]:
            for n, (_, t) in enumerate(r["proposed"]):
                want[r["step"], n] = t
            if not r["accepted"]:
                assert list(own_t[b, r["step"], :len(r["final_tokens"])]) == r["final_tokens"]
            if sampled:                      # the acceptance tests up to and including each round's first refusal
                n0 = 0
                for made, kept in r["sd_rounds"]:
                    assert list(flags[b, r["step"], n0:n0 + kept]) == [1] * kept, (b, r["step"], n0)
                    if kept < made:
                        assert flags[b, r["step"], n0 + kept] == 0
                    n0 += made
        assert np.array_equal(prop[b], want), b
    st = R.rsd_export_state(s.ctx)
    for b in range(w.batch):
        n = st["ctx_len"][b]
        assert b in skip or list(st["tokens"][b, :n]) == refs[b]["tokens"][:n]
    s.close()
    return tot


@pytest.mark.parametrize("sd_k", [1, 3, 7])
def test_config0_regeneration_by_speculation(gpu, tiny, sd_k):
    from rsd_inputs import workload
    w = workload("cfg0", sep_logit_bias=0.6, deltas=(0.55,))
    tot = compare_sd(gpu, w, tiny["models"], sd_k)
    assert tot["rej"] >= 2 and tot["rounds"] > 0 and tot["prop"] >= tot["rounds"] - tot["rej"]
    print(tot)


@pytest.mark.parametrize("merge", [1, 2])
def test_config0_speculation_with_merged_reward_head(gpu, tiny, merge):
    from rsd_inputs import workload, model_weights_np
    from oracle import rsd_oracle as O
    w = workload("cfg0", sep_logit_bias=0.6)
    policy = w.draft if merge == 1 else w.target
    w = replace(w, prm=replace(policy, head_kind="reward"))
    head = model_weights_np(w.seed, 2, w.prm)
    trunk = tiny["models"][merge - 1]._w
    pm = O.OracleModel(w.prm, {**{k: v for k, v in trunk.items() if k != "lm_head"}, "w_r": head["w_r"], "b_r": head["b_r"]})
    models = [tiny["models"][0], tiny["models"][1], pm]
    w = replace(w, deltas=(1.01,))                # every step rejected
    tot = compare_sd(gpu, w, models, 3, merge=merge)
    assert tot["rej"] >= 8


def test_a_draft_equal_to_the_target_has_every_proposal_kept(gpu, tiny):
    """Two copies of one model: every proposal is kept, rounds commit sd_k + 1 tokens, and the draft
    then has two tokens to catch up with (its chunked path inside the proposal stage)."""
    from rsd_inputs import workload, model_blob_torch
    import torch
    w = workload("cfg0", sep_logit_bias=0.3, deltas=(1.01,))
    w = replace(w, draft=w.target)
    d, t, p = tiny["models"]
    dev = torch.device("cuda:0")
    blobs = [model_blob_torch(w.seed, 1, w.target, dev), model_blob_torch(w.seed, 1, w.target, dev),
             model_blob_torch(w.seed, 2, w.prm, dev)]
    tot = compare_sd(gpu, w, [t, t, p], 3, weights=blobs)
    assert tot["prop"] == tot["kept"] > 0


def test_a_draft_close_to_the_target_has_some_proposals_kept(gpu, tiny):
    """The draft is the target with a perturbed output head: rounds end at every place from the first
    proposal to the extra token, and the draft's cache is cut back by a different amount each time."""
    from rsd_inputs import workload, model_blob_np, model_blob_torch, weights_from_blob
    from oracle import rsd_oracle as O
    import torch
    w = workload("cfg0", sep_logit_bias=0.6, deltas=(1.01,), max_steps=3)
    w = replace(w, draft=w.target)
    blob = model_blob_np(w.seed, 1, w.target).copy()
    wd = weights_from_blob(blob, w.target)
    r = np.random.default_rng(4)
    wd["lm_head"] += (0.012 * r.standard_normal(wd["lm_head"].shape)).astype(np.float32)    # views: edits the blob
    dm = O.OracleModel(w.draft, wd)
    d, t, p = tiny["models"]
    dev = torch.device("cuda:0")
    blobs = [torch.from_numpy(blob).to(dev), model_blob_torch(w.seed, 1, w.target, dev), model_blob_torch(w.seed, 2, w.prm, dev)]
    tot = compare_sd(gpu, w, [dm, t, p], 4, weights=blobs, min_margin=5e-5)
    print(tot)
    assert tot["skipped"] <= 1 and 0.05 * tot["prop"] < tot["kept"] < 0.9 * tot["prop"]


def test_speculation_leaves_the_committed_tokens_unchanged(gpu, tiny):
    """Greedy: with and without speculation the HIP path commits the same tokens."""
    from rsd_inputs import workload
    R = gpu["R"]
    w = workload("cfg0", sep_logit_bias=0.6, deltas=(0.55,))
    outs = []
    for k in (0, 5):
        s = gpu["Session"](w, sd_k=k)
        outs.append(R.rsd_generate(s.ctx))
        s.close()
    a, b = outs
    assert np.array_equal(a["ctx_len"], b["ctx_len"])
    for i in range(w.batch):
        assert np.array_equal(a["tokens"][i, :a["ctx_len"][i]], b["tokens"][i, :b["ctx_len"][i]])
    assert a["n_sd_rounds"] == 0 and b["n_sd_rounds"] > 0 and b["n_sd_proposed"] >= b["n_sd_kept"]


@pytest.mark.parametrize("sd_k,top_p", [(3, 0.95), (6, 1.0), (2, 0.6)])
def test_config0_sampled_speculation(gpu, tiny, sd_k, top_p):
    """Temperature / nucleus sampling: proposals drawn from the draft's distribution, kept with
    probability min(1, p/q), replaced by a draw from the positive part of p - q."""
    from rsd_inputs import workload
    w = workload("cfg0", sep_logit_bias=3.5, deltas=(0.55,), temperature=0.7, top_p=top_p)
    tot = compare_sd(gpu, w, tiny["models"], sd_k)
    print(tot)
    assert tot["rej"] >= 2 and 0 < tot["kept"] < tot["prop"]


def _tight(w, max_ctx):
    """The same workload with a context limit below prompt + steps x cap, so that sequences fill up mid-step."""
    from dataclasses import fields

    class Tight(type(w)):
        @property
        def max_ctx(self):
            return max_ctx

    return Tight(**{f.name: getattr(w, f.name) for f in fields(w)})


@pytest.mark.parametrize("case", ["cap1", "cap2", "eos_sampled", "ctx_greedy", "ctx_sampled"])
def test_speculation_edge_cases(gpu, tiny, case):
    """One-token steps (no room for a proposal: every round is a plain target token), two-token steps (one
    proposal), EOS among proposals and committed tokens, and a context that fills up in the middle of a
    round (the proposal budget shrinks to what the context leaves after the target's own token)."""
    from rsd_inputs import workload
    if case == "cap1":
        w, k = workload("cfg0", step_cap=1, max_steps=6, deltas=(1.01,)), 3
    elif case == "cap2":
        w, k = workload("cfg0", step_cap=2, max_steps=6, deltas=(1.01,), temperature=0.7, top_p=0.95), 3
    elif case == "eos_sampled":
        w, k = workload("cfg0", sep_logit_bias=3.5, deltas=(0.55,), temperature=0.7, top_p=0.95, eos_id=517, max_steps=5), 3
    elif case == "ctx_greedy":
        w, k = _tight(workload("cfg0", sep_logit_bias=0.6, deltas=(1.01,)), 32 + 37), 5
    else:
        w, k = _tight(workload("cfg0", sep_logit_bias=2.0, deltas=(1.01,), temperature=0.7, top_p=0.95), 32 + 27), 4
    tot = compare_sd(gpu, w, tiny["models"], k)
    print(case, tot)
    assert tot["rej"] >= 2
    if case == "cap1":
        assert tot["prop"] == 0 and tot["rounds"] == tot["rej"]


def test_speculation_replayed_from_graphs_matches_eager_launches(gpu):
    """The proposal iterations are replayed from their own recorded graph (the append works in its
    "proposal" flavour there, and under sampling a copy of the draft's logits is part of the graph):
    same kernels as the kernel-by-kernel run, so everything must agree bit for bit."""
    from rsd_inputs import workload
    R = gpu["R"]
    w = workload("cfg0", sep_logit_bias=3.5, deltas=(0.55,), temperature=0.7, top_p=0.95)
    outs = []
    for use_graphs in (0, 1):
        s = gpu["Session"](w, sd_k=4, use_graphs=use_graphs)
        g = R.rsd_generate(s.ctx)
        st = R.rsd_decode_stats(s.ctx)
        outs.append((g, R.rsd_export_proposed(s.ctx, want_flags=True), st))
        s.close()
    (a, pa, sa), (b, pb, sb) = outs
    assert sa["graph_replays"] == 0 and sb["graph_replays"] > 0 and sb["graphs_recorded"] >= 2
    assert np.array_equal(a["tokens"], b["tokens"]) and np.array_equal(a["ctx_len"], b["ctx_len"])
    assert np.array_equal(pa[0], pb[0]) and np.array_equal(pa[1], pb[1])
    assert (a["n_sd_rounds"], a["n_sd_proposed"], a["n_sd_kept"]) == (b["n_sd_rounds"], b["n_sd_proposed"], b["n_sd_kept"])
    assert a["n_sd_kept"] > 0


def test_sampled_verification_rule_alone(gpu):
    """rsd_sd_verify on given logits against the checker's rule on the same fp32 logits: kept counts and
    emitted tokens, over cases with 0..sd_k proposals, drafts close to and far from the target, equal rows
    (all kept) and a sharply peaked target."""
    from oracle import rsd_oracle as O
    from rsd_inputs import workload
    R, torch = gpu["R"], gpu["torch"]
    k, T, top_p, bias = 4, np.float32(0.8), np.float32(0.9), np.float32(1.5)
    w = workload("cfg0", temperature=float(T), top_p=float(top_p), sep_logit_bias=float(bias))
    s = gpu["Session"](w, sd_k=k)
    V, n = w.draft.vocab, w.batch
    rng = np.random.default_rng(21)
    n_case = n_excused = 0
    kept_hist = np.zeros(k + 1, int)
    for call in range(30):
        p = (rng.normal(size=(n, k + 1, V)) * 2.0).astype(np.float32)
        mix = rng.choice([0.0, 0.3, 1.0, 3.0], size=(n, 1, 1)).astype(np.float32)
        q = (p[:, :k] + mix * rng.normal(size=(n, k, V)).astype(np.float32)).astype(np.float32)
        if call % 5 == 0:
            p[0, :, 7] += 12.0                                    # a peaked target row set
        cnt = rng.integers(0, k + 1, size=n).astype(np.int32)
        u_acc = rng.random((n, k + 1)).astype(np.float32)
        u_new = rng.random((n, k + 1)).astype(np.float32)
        u_draw = rng.random((n, k))

        def dist(lg):
            x = lg.astype(np.float64).copy()
            x[w.sep_id] += float(bias)
            return O.token_distribution(x, float(T), float(top_p))

        props = np.zeros((n, k), np.int32)
        for c in range(n):
            for i in range(k):
                props[c, i] = O.draw(dist(q[c, i]), u_draw[c, i])
        dev = lambda a: torch.from_numpy(a).cuda()
        em, kept = R.rsd_sd_verify(s.ctx, dev(p), dev(q), dev(props), cnt, dev(u_acc), dev(u_new))
        for c in range(n):
            g = int(cnt[c])
            q_rows = [dist(q[c, i]) for i in range(g)]
            p_rows = [dist(p[c, i]) for i in range(g + 1)]
            want, wkept = O.sd_verify(q_rows, p_rows, list(props[c, :g]), list(u_acc[c, :g]), list(u_new[c, :g + 1]))
            n_case += 1
            # a decision within 1e-5 (relative) of its threshold may fall either way in fp32
            close = any(abs(float(u_acc[c, i]) * q_rows[i][props[c, i]] - p_rows[i][props[c, i]]) < 1e-5 * q_rows[i][props[c, i]]
                        for i in range(min(g, wkept + 1)))
            if close and (kept[c] != wkept or list(em[c, :wkept + 1]) != want):
                n_excused += 1
                continue
            assert kept[c] == wkept, (call, c, kept[c], wkept)
            assert list(em[c, :wkept + 1]) == want, (call, c, list(em[c]), want)
            kept_hist[wkept] += 1
    print("cases", n_case, "excused", n_excused, "kept histogram", kept_hist)
    assert n_excused <= 2 and np.all(kept_hist[:k] > 0) and kept_hist[k] > 0
    s.close()


# ------------------------------------------------------------------ bf16, under a teacher
def _bf16_setup(gpu, batch, sd_k, check, **kw):
    import test_gpu_bf16 as T
    from oracle import rsd_oracle as O
    R, torch = gpu["R"], gpu["torch"]
    w = T.mid_workload(batch, **kw)
    models = T.oracle_models(T.mid_workload(3))
    s = gpu["Session"](w, sd_k=sd_k)
    P = replace(T.oracle_params(O, w), sd_k=sd_k)
    sampled = w.temperature > 0
    refs = {b: O.generate_sequence(*models, s.tokens_host[b, :s.prompt_len[b]], s.u_host["U_DRAFT"][b],
                                   s.u_host["U_TARGET"][b], s.u_host["U_GATE"][b], P,
                                   u_prop=s.u_host["U_PROP"][b] if sampled else None,
                                   u_acc=s.u_host["U_ACC"][b] if sampled else None, keep_draws=sampled) for b in check}
    allrefs = [refs.get(b, dict(records=[])) for b in range(w.batch)]
    forced, _ = T.teacher_arrays(w, allrefs, torch)
    fp = np.full((w.batch, w.max_steps, w.step_cap * sd_k), -1, np.int32)
    for b, ref in refs.items():
        for r in ref["records"]:
            for n, (_, t) in enumerate(r["proposed"]):
                fp[b, r["step"], n] = t
    fp_dev = torch.from_numpy(fp).cuda()
    R.rsd_set_teacher(s.ctx, *forced)
    R.rsd_set_teacher_sd(s.ctx, fp_dev)
    s.reset()
    s.checker_models = models
    return w, s, refs


# ---- when may a random decision of the HIP path differ from the checker's?  Only where the error of the
# logits it was taken on (measured in the same test, on the same trajectory) can move it: a logit error of
# eps changes the ratio of two tokens' probabilities by at most exp(2 eps / T) - 1 =: f, hence every point of
# a nucleus distribution function by at most f plus the mass of the tokens whose membership in the nucleus it
# can flip (probability within a factor exp(+-2 eps / T) of the threshold).
def _nucleus(O, lg, temp, top_p, eps):
    p = O.softmax(np.asarray(lg) / temp)
    order = np.argsort(-p, kind="stable")
    cum = np.cumsum(p[order])
    reach = np.nonzero(cum >= top_p)[0]
    tau = p[order[reach[0]]] if reach.size else np.min(p)
    a = 2.0 * eps / temp
    band = float(np.sum(p[(p >= tau * np.exp(-a)) & (p <= tau * np.exp(a))]))
    keep = p >= tau
    return p, keep, float(np.sum(p[keep])), np.exp(a) - 1.0, band


def _cdf_distance(dist, u, tok):
    """Distance (in probability) from the point the uniform u marks to the interval token `tok` occupies in
    the distribution function of `dist` walked in ascending token id."""
    z = float(np.sum(dist))
    lo = float(np.sum(dist[:tok])) / z
    hi = lo + float(dist[tok]) / z
    return max(0.0, lo - u, u - hi)


def _draw_in_reach(O, e, tok, temp, top_p, eps_d, eps_t):
    if e["kind"] in ("prop", "tgt"):
        eps = eps_d if e["kind"] == "prop" else eps_t
        p, keep, z, f, band = _nucleus(O, e["lg"], temp, top_p, eps)
        return _cdf_distance(np.where(keep, p, 0.0), e["u"], tok) <= f + 3.0 * band / z
    pp, kp, zp, fp_, bp = _nucleus(O, e["lg_p"], temp, top_p, eps_t)
    pq, kq, zq, fq, bq = _nucleus(O, e["lg_q"], temp, top_p, eps_d)
    res = np.maximum(np.where(kp, pp, 0.0) / zp - np.where(kq, pq, 0.0) / zq, 0.0)
    zr = float(np.sum(res))
    return zr == 0.0 or _cdf_distance(res, e["u"], tok) <= min(1.0, (2 * fp_ + 2 * fq + 3 * (bp / zp + bq / zq)) / zr)


def _flag_in_reach(O, e, temp, top_p, eps_d, eps_t):
    pp, kp, zp, fp_, bp = _nucleus(O, e["lg_p"], temp, top_p, eps_t)
    pq, kq, zq, fq, bq = _nucleus(O, e["lg_q"], temp, top_p, eps_d)
    x = e["tok"]
    a_t, a_d = np.log1p(fp_), np.log1p(fq)
    tau_p, tau_q = np.min(pp[kp]), np.min(pq[kq])
    if tau_p * np.exp(-a_t) <= pp[x] <= tau_p * np.exp(a_t) or tau_q * np.exp(-a_d) <= pq[x] <= tau_q * np.exp(a_d):
        return True                                   # the proposal's membership in a nucleus can flip
    px = pp[x] / zp if kp[x] else 0.0
    qx = pq[x] / zq if kq[x] else 0.0
    return abs(px - e["u"] * qx) <= (2 * fp_ + 3 * bp / zp) * px + (2 * fq + 3 * bq / zq) * e["u"] * qx


def _measured_logit_error(gpu, w, s, refs, models):
    """Largest error of the HIP path's draft and target logits along the committed trajectories."""
    from oracle import rsd_oracle as O
    R = gpu["R"]
    T_ = max(len(ref["tokens"]) for ref in refs.values())
    toks = np.zeros((w.batch, T_), np.int32)
    lens = np.zeros(w.batch, np.int32)
    for b, ref in refs.items():
        lens[b] = len(ref["tokens"])
        toks[b, :lens[b]] = ref["tokens"]
    worst = []
    for which in (0, 1):
        out = R.rsd_forward(s.ctx, which, toks, lens, 1)
        err = 0.0
        for b, ref in refs.items():
            lg = O.lm_logits(models[which], O.forward_full(models[which], ref["tokens"], "bf16"))
            err = max(err, float(np.max(np.abs(out[b, :lens[b]].cpu().numpy() - lg))))
        worst.append(err)
    return worst


def _bf16_follow(gpu, w, s, refs):
    import test_gpu_bf16 as T
    from oracle import rsd_oracle as O
    R = gpu["R"]
    models = s.checker_models
    tot = dict(rej=0, rounds=0, prop=0, kept=0, excused=0, tokens=0)
    for i in range(w.max_steps):
        g = R.rsd_step(s.ctx)
        st = R.rsd_export_state(s.ctx, want_tokens=False)
        for b, ref in refs.items():
            r = ref["records"][i]
            assert abs(float(g["reward"][b]) - r["reward"]) < T.TOL
            assert bool(g["accepted"][b]) == r["accepted"]
            assert list(g["final_tokens"][b, :g["final_len"][b]]) == r["final_tokens"]
            assert list(st["kv_len"][:, b]) == r["kv_len"], (b, i, list(st["kv_len"][:, b]), r["kv_len"])
            assert list(st["n_pages"][:, b]) == r["n_pages"] and st["ctx_len"][b] == r["ctx_len"]
            rounds = r["sd_rounds"]
            want = (len(rounds), sum(p for p, _ in rounds), sum(k for _, k in rounds))
            assert (g["sd_rounds"][b], g["sd_proposed"][b], g["sd_kept"][b]) == want, (b, i, rounds)
            tot["rej"] += not r["accepted"]; tot["rounds"] += len(rounds)
            tot["prop"] += sum(p for p, _ in rounds); tot["kept"] += sum(k for _, k in rounds)
        for b in range(w.batch):                       # the offset contract holds for every sequence
            kd, kt, kp = (int(v) for v in st["kv_len"][:, b])
            ctx = int(st["ctx_len"][b])
            if g["accepted"][b]:
                assert kd == ctx - 1 and kp == ctx and g["sd_rounds"][b] == 0
            elif g["final_len"][b]:
                assert kt == ctx - 1 and kd <= ctx - 1 and kp == ctx - int(g["final_len"][b])
                assert 0 <= g["sd_kept"][b] <= g["sd_proposed"][b] and g["sd_rounds"][b] >= 1
    # the models' own choices.  Greedy: equal to the checker's except at near-ties of the logits.  Sampled:
    # a differing draw or acceptance test must lie within the reach of the logits' measured error (see above)
    sampled = w.temperature > 0
    prop, flags = R.rsd_export_proposed(s.ctx, want_flags=True)
    _, own_t = R.rsd_export_sampled(s.ctx)
    R.rsd_set_teacher(s.ctx, None, None, None)
    R.rsd_set_teacher_sd(s.ctx, None)
    eps_d = eps_t = 0.0
    if sampled:
        eps_d, eps_t = _measured_logit_error(gpu, w, s, refs, models)
        assert eps_d < T.TOL and eps_t < T.TOL
        tot["logit_error"] = (round(eps_d, 5), round(eps_t, 5))
        eps_d, eps_t = 2 * eps_d, 2 * eps_t        # draws inside a round are taken on contexts with proposals: allow twice the measured error
    temp, top_p = float(np.float32(w.temperature)), float(np.float32(w.top_p))
    for b, ref in refs.items():
        for r in ref["records"]:
            dr = r.get("draws") or []
            props = [e for e in dr if e["kind"] == "prop"]
            for n, ((j, t), gap) in enumerate(zip(r["proposed"], r["proposal_margins"])):
                tot["tokens"] += 1
                mine = int(prop[b, r["step"], n])
                if mine != t:
                    if sampled:
                        assert props[n]["tok"] == t
                        assert _draw_in_reach(O, props[n], mine, temp, top_p, eps_d, eps_t), (b, r["step"], n, mine, t)
                    else:
                        assert gap < 2 * T.TOL, (b, r["step"], n, j, gap)
                    tot["excused"] += 1
            if not r["accepted"]:
                own_draws = {e["place"]: e for e in dr if e["kind"] in ("res", "tgt")}
                for j, (t, gap) in enumerate(zip(r["final_tokens"], r["final_margins"])):
                    tot["tokens"] += 1
                    mine = int(own_t[b, r["step"], j])
                    if mine != t:
                        if sampled:
                            e = own_draws[j]         # kept proposals are copied, so only the target's own draws can differ
                            assert e["tok"] == t
                            assert _draw_in_reach(O, e, mine, temp, top_p, eps_d, eps_t), (b, r["step"], j, mine, t)
                        else:
                            assert gap < 2 * T.TOL, (b, r["step"], j, gap)
                        tot["excused"] += 1
            if sampled:
                accs = [e for e in dr if e["kind"] == "acc"]
                n0 = a0 = 0
                for made, kept in r["sd_rounds"]:
                    want = [1] * kept + ([0] if kept < made else [])
                    got = list(flags[b, r["step"], n0:n0 + len(want)])
                    tot["tokens"] += len(want)
                    for i, (x, y) in enumerate(zip(got, want)):
                        e = accs[a0 + i]
                        assert e["kept"] == bool(y)
                        if x != y:
                            assert _flag_in_reach(O, e, temp, top_p, eps_d, eps_t), (b, r["step"], n0 + i)
                            tot["excused"] += 1
                    n0 += made
                    a0 += len(want)
    R.rsd_set_teacher(s.ctx, None, None, None)
    R.rsd_set_teacher_sd(s.ctx, None)
    s.close()
    return tot


@pytest.mark.parametrize("batch,sd_k", [(1, 7), (3, 3), (12, 2)])
def test_teacher_forced_speculation_bf16(gpu, batch, sd_k):
    """Batch 1 and 3: the verification rows go through the weight-streaming kernels (<= 8 rows) or the
    few-row MFMA GEMM; batch 12: more rows."""
    check = list(range(min(batch, 3)))
    w, s, refs = _bf16_setup(gpu, batch, sd_k, check, step_cap=10)
    tot = _bf16_follow(gpu, w, s, refs)
    print(tot)
    assert tot["rej"] >= 1 and tot["rounds"] > 0 and tot["excused"] <= max(2, tot["tokens"] // 10)


@pytest.mark.parametrize("batch,sd_k", [(1, 5), (3, 3)])
def test_teacher_forced_sampled_speculation_bf16(gpu, batch, sd_k):
    """Top-p sampling (T = 0.7, p = 0.95) in bf16 under a teacher for the target's tokens and the
    proposals: committed tokens, counts and offsets exact; each of the path's own draws and acceptance
    tests that differs from the checker's must lie within the reach of the logits' measured error (the
    distance of the uniform to the token's interval of the distribution function, or of u q(x) to p(x));
    the number of such cases is printed."""
    check = list(range(min(batch, 3)))
    w, s, refs = _bf16_setup(gpu, batch, sd_k, check, step_cap=10, temperature=0.7, top_p=0.95, sep_logit_bias=4.0,
                             deltas=(0.62,))
    tot = _bf16_follow(gpu, w, s, refs)
    print(tot)
    assert tot["rej"] >= 1 and tot["kept"] > 0          # (every differing draw was judged on its own in _bf16_follow)


def test_large_batch_speculation_bf16(gpu):
    """64 sequences with prompts of up to 400 tokens: the target's first verification pass would exceed
    one prefill pass, so the unseen prefixes are read first (several passes) and the proposals after."""
    batch = 64
    check = [0, 31, 63]
    w, s, refs = _bf16_setup(gpu, batch, 4, check, prompt_len_min=16, prompt_len_max=400, step_cap=8, max_steps=3,
                             deltas=(0.75,))
    tot = _bf16_follow(gpu, w, s, refs)
    print(tot)
    assert tot["rej"] >= 1
