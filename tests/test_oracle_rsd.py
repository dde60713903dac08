"""Pins of the CPU checker's decoding loop, sampler and acceptance criterion:
fixed points of the gate, values printed in the paper, closed forms and
brute force."""
import os

import numpy as np
import pytest

from oracle import rsd_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")
# settings under which the tiny random-init models end steps early and the gate
# both accepts and rejects (found by looking at the checker's own rewards)
GREEDY_MIX = dict(sep_logit_bias=0.6, delta=0.55)
SAMPLED_MIX = dict(temperature=0.7, top_p=0.95, sep_logit_bias=3.5, delta=0.55)


def params(w, **kw):
    base = dict(delta=w.delta, sep_id=w.sep_id, step_cap=w.step_cap, max_steps=w.max_steps,
                max_ctx=w.max_ctx, eos_id=w.eos_id, temperature=w.temperature, top_p=w.top_p,
                sep_logit_bias=w.sep_logit_bias)
    base.update(kw)
    return O.Params(**base)


def run(tiny, b, P, use_cache=True, models=None, **kw):
    d, t, p = models or tiny["models"]
    return O.generate_sequence(d, t, p, tiny["tokens"][b, :tiny["lens"][b]], tiny["u_draft"][b],
                               tiny["u_target"][b], tiny["u_gate"][b], P, use_cache=use_cache, **kw)


# ------------------------------------------------------------ gate fixed points
@pytest.mark.parametrize("temperature,top_p,bias", [(0.0, 1.0, 0.0), (0.0, 1.0, 0.6), (0.7, 0.95, 3.5)])
def test_delta_below_zero_is_draft_only_and_above_one_is_target_only(tiny, temperature, top_p, bias):
    """delta <= 0 accepts every step, delta > 1 rejects every step (the reward
    lies in [0, 1]); the committed tokens then equal ordinary decoding with
    the draft, respectively the target, computed here with no cache and no
    notion of steps."""
    w = tiny["w"]
    for b in (0, 3):
        prompt = tiny["tokens"][b, :tiny["lens"][b]]
        for delta, which, u in ((0.0, 0, "u_draft"), (-1.0, 0, "u_draft"), (1.01, 1, "u_target")):
            P = params(w, delta=delta, temperature=temperature, top_p=top_p, sep_logit_bias=bias, max_steps=3)
            out = run(tiny, b, P)
            gen = out["tokens"][len(prompt):]
            ref = O.decode_plain(tiny["models"][which], prompt, tiny[u][b], P, len(gen))
            assert gen == ref
            assert all(r["accepted"] == (which == 0) for r in out["records"])
            if which == 0:
                assert out["kv_len"][1] == 0            # the target was never touched
    if bias:
        lens = [len(r["final_tokens"]) for r in out["records"]]
        assert min(lens) < w.step_cap                   # separators did end steps early


def test_threshold_is_inclusive(tiny):
    """A reward head of all zeros gives r = 1/2 exactly: delta = 1/2 accepts
    every step (r >= delta, Table 1), the next float above rejects every one."""
    d, t, p0 = tiny["models"]
    w = {k: np.array(v, copy=True) for k, v in p0._w.items()}
    w["w_r"][:] = 0
    p = O.OracleModel(p0.s, w)
    up = float(np.nextafter(np.float32(0.5), np.float32(1.0)))
    a = run(tiny, 1, params(tiny["w"], delta=0.5, max_steps=2), models=(d, t, p))
    r = run(tiny, 1, params(tiny["w"], delta=up, max_steps=2), models=(d, t, p))
    assert all(x["reward"] == 0.5 and x["accepted"] for x in a["records"])
    assert all(x["reward"] == 0.5 and not x["accepted"] for x in r["records"])


def test_cache_and_no_cache_runs_agree(tiny):
    """Incremental KV with rollback and lazy target catch-up against a run that
    recomputes the whole prefix for every token."""
    seen = set()
    for b in range(tiny["w"].batch):
        P = params(tiny["w"], **(GREEDY_MIX if b % 2 else SAMPLED_MIX))
        a = run(tiny, b, P, use_cache=True)
        c = run(tiny, b, P, use_cache=False)
        assert a["tokens"] == c["tokens"]
        for ra, rc in zip(a["records"], c["records"]):
            assert ra["draft_tokens"] == rc["draft_tokens"] and ra["accepted"] == rc["accepted"]
            assert abs(ra["reward"] - rc["reward"]) < 1e-12
            assert ra["kv_len"] == rc["kv_len"]
            seen.add(ra["accepted"])
    assert seen == {True, False}


def test_cache_and_no_cache_runs_agree_with_bf16_storage(tiny):
    P = params(tiny["w"], kv_dtype="bf16", **GREEDY_MIX)
    for b in (1, 3):
        a = run(tiny, b, P, use_cache=True)
        c = run(tiny, b, P, use_cache=False)
        assert a["tokens"] == c["tokens"]
        assert [r["accepted"] for r in a["records"]] == [r["accepted"] for r in c["records"]]
        assert max(abs(x["reward"] - y["reward"]) for x, y in zip(a["records"], c["records"])) < 1e-12


def test_kv_offsets_follow_the_contract(tiny):
    """After a step: accepted -> draft holds ctx-1 tokens, reward model ctx,
    target unchanged; rejected -> draft and reward model hold the pre-step
    context, target ctx-1."""
    n_rej = 0
    for b in range(tiny["w"].batch):
        P = params(tiny["w"], **(GREEDY_MIX if b % 2 else SAMPLED_MIX))
        out = run(tiny, b, P)
        n_rej += sum(not r["accepted"] for r in out["records"])
        kv_t_prev = 0
        for r in out["records"]:
            kd, kt, kp = r["kv_len"]
            if r["accepted"]:
                assert (kd, kt, kp) == (r["ctx_len"] - 1, kv_t_prev, r["ctx_len"])
            else:
                assert (kd, kt, kp) == (r["ctx_pre"], r["ctx_len"] - 1, r["ctx_pre"])
            assert r["n_pages"] == [-(-n // 16) for n in r["kv_len"]]
            assert r["ctx_len"] == r["ctx_pre"] + len(r["final_tokens"])
            kv_t_prev = kt
    assert n_rej >= 2


def test_eos_stops_generation_only_when_committed(tiny):
    """Declare, in turn, each token of a baseline run to be EOS.  A step stops
    right after an EOS; the sequence finishes only when a committed step holds
    it; an EOS inside a rejected draft step is thrown away with that step."""
    w = tiny["w"]
    base = run(tiny, 0, params(w, **SAMPLED_MIX))
    cands = sorted({t for r in base["records"] for t in r["draft_tokens"] + r["final_tokens"]} - {w.sep_id})
    saw_finish = saw_discard = 0
    for eos in cands[:24]:
        out = run(tiny, 0, params(w, eos_id=eos, **SAMPLED_MIX))
        recs = out["records"]
        for r in recs:
            for step in (r["draft_tokens"], r["final_tokens"]):
                assert eos not in step[:-1]
        for r in recs[:-1]:
            assert eos not in r["final_tokens"]
        if eos in recs[-1]["final_tokens"]:
            assert out["finished"] == O.FIN_EOS
            saw_finish += 1
        else:
            assert out["finished"] == O.FIN_MAX_STEPS and len(recs) == w.max_steps
        for k, r in enumerate(recs):
            if not r["accepted"] and r["draft_tokens"][-1] == eos and r["final_tokens"][-1] != eos:
                saw_discard += 1
    assert saw_finish >= 1 and saw_discard >= 1


def test_context_limit(tiny):
    w = tiny["w"]
    out = run(tiny, 2, params(w, max_ctx=32 + 21))
    assert out["finished"] == O.FIN_MAX_CTX and len(out["tokens"]) == 53
    assert [len(r["final_tokens"]) for r in out["records"]] == [16, 5]


# ------------------------------------------------------------ sampler
def nucleus_textbook(p, top_p):
    """Sort-based nucleus: smallest set of most probable tokens whose mass
    reaches top_p (no ties in these tests)."""
    order = np.argsort(-p)
    n = int(np.searchsorted(np.cumsum(p[order]), top_p, side="left")) + 1
    keep = np.zeros(p.size, bool)
    keep[order[:n]] = True
    return keep


def test_greedy_takes_lowest_id_on_ties():
    lg = np.array([0.1, 2.0, -1.0, 2.0, 0.5])
    assert O.sample(lg, 0.9, 0.0, 1.0) == 1
    assert O.sample(lg, 0.1, 0.0, 0.3) == 1


def test_top_p_one_is_inverse_cdf_and_small_settings_are_greedy():
    r = np.random.default_rng(0)
    lg = r.normal(size=200) * 2
    p = O.softmax(lg / 0.7)
    cdf = np.cumsum(p)
    for u in r.random(500):
        assert O.sample(lg, u, 0.7, 1.0) == int(np.searchsorted(cdf, u * cdf[-1], side="right"))
    for u in (0.0, 0.3, 0.999):
        assert O.sample(lg, u, 0.7, 1e-9) == int(np.argmax(lg))
        assert O.sample(lg, u, 1e-4, 0.95) == int(np.argmax(lg))


def test_nucleus_frequencies():
    r = np.random.default_rng(1)
    lg = r.normal(size=50) * 1.5
    T, top_p = 0.7, 0.8
    p = O.softmax(lg / T)
    keep = nucleus_textbook(p, top_p)
    q = np.where(keep, p, 0.0)
    q /= q.sum()
    n = 100000
    us = (np.arange(n) + 0.5) / n                       # stratified uniforms
    draws = np.array([O.sample(lg, u, T, top_p) for u in us])
    freq = np.bincount(draws, minlength=50) / n
    assert set(np.nonzero(freq)[0]) == set(np.nonzero(keep)[0])
    assert np.max(np.abs(freq - q)) < 2.0 / n + 1e-12


def test_nucleus_keeps_boundary_ties_and_walks_ids_upwards():
    p = np.array([0.1, 0.3, 0.1, 0.3, 0.1, 0.1])
    lg = np.log(p)
    # mass of {p >= 0.3} = 0.6 >= 0.5: nucleus {1, 3}; both boundary ties stay
    assert [O.sample(lg, u, 1.0, 0.5) for u in (0.0, 0.49, 0.51, 0.99)] == [1, 1, 3, 3]
    # top_p 0.7 needs the 0.1 level: every token of that level joins
    assert sorted({O.sample(lg, u, 1.0, 0.7) for u in np.linspace(0, 0.999, 400)}) == [0, 1, 2, 3, 4, 5]
    # u * Z exactly on an edge moves to the next token ("exceeds")
    p2 = np.array([0.25, 0.25, 0.5])
    assert O.sample(np.log(p2), 0.25, 1.0, 1.0) == 1 and O.sample(np.log(p2), 0.5, 1.0, 1.0) == 2


# ------------------------------------------------------------ acceptance criterion
def test_weighting_functions_table():
    assert [O.omega(r, O.OMEGA_BINARY, 0.7) for r in (0.69, 0.7, 0.71)] == [0.0, 1.0, 1.0]
    assert O.omega(0.2, O.OMEGA_CONSTANT, 0.7, 0.6) == 0.6
    assert [O.omega(r, O.OMEGA_CLIP, 0.0) for r in (-0.5, 0.25, 3.0)] == [0.0, 0.25, 1.0]
    assert O.omega(1.0, O.OMEGA_RATIO, 0.0) == 0.5 and O.omega(-0.5, O.OMEGA_RATIO, 0.0) == 0.0
    assert O.omega(0.6, O.OMEGA_LOGISTIC, 0.6, 1.0) == 0.5
    assert abs(O.omega(1.6, O.OMEGA_LOGISTIC, 0.6, 2.0) - 1 / (1 + np.exp(-2.0))) < 1e-15


def test_criterion_is_deterministic_at_zero_and_one_and_random_between():
    for u in (0.0, 0.5, 0.999999):
        assert O.accept(0.7, O.OMEGA_BINARY, 0.7, 0.0, u) is True
        assert O.accept(0.69, O.OMEGA_BINARY, 0.7, 0.0, u) is False
        assert O.accept(1.5, O.OMEGA_CLIP, 0.0, 0.0, u) is True       # weight exactly 1
        assert O.accept(-0.1, O.OMEGA_CLIP, 0.0, 0.0, u) is False     # weight exactly 0, even for u = 0
    us = (np.arange(10000) + 0.5) / 10000
    assert abs(np.mean([O.accept(0.3, O.OMEGA_CLIP, 0.0, 0.0, u) for u in us]) - 0.3) < 1e-3
    assert abs(np.mean([O.accept(0.0, O.OMEGA_CONSTANT, 0.0, 0.6, u) for u in us]) - 0.6) < 1e-3


def test_figure_2_normalising_constant():
    """The illustration of the mixture (Section 2, Fig. 2) draws P_m and P_M as
    Gaussians of means 0 and 2, the weight N(r;1.5,1)/(N(r;0,1)+N(r;1.5,1)),
    and prints nu as 1 - 1.16/3.77.  Discretise the line finely and let the
    checker's mixture function produce nu."""
    vals = {}
    for line in open(os.path.join(GOLD, "fig2_mixture.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            vals[k] = float(v)
    x = np.linspace(-12, 14, 260001)
    dx = x[1] - x[0]
    g = lambda mu: np.exp(-0.5 * (x - mu) ** 2)
    w = g(1.5) / (g(0.0) + g(1.5))
    mass_m = np.sum(vals["amplitude"] * g(0.0)) * dx
    mass_wm = np.sum(w * vals["amplitude"] * g(0.0)) * dx
    assert abs(mass_m - vals["mass_pm_printed"]) < 0.015           # printed to 2 decimals
    assert abs(mass_wm - vals["mass_wpm_printed"]) < 0.01
    p_m = g(0.0) / np.sum(g(0.0))
    p_M = g(2.0) / np.sum(g(2.0))
    mix, nu = O.mixture_distribution(p_m, p_M, w)
    assert abs(nu - (1 - vals["mass_wpm_printed"] / vals["mass_pm_printed"])) < 0.005
    assert abs(np.sum(mix) - 1.0) < 1e-12
    assert abs(nu - (1 - mass_wm / mass_m)) < 1e-12


@pytest.mark.parametrize("kind,a,delta", [(O.OMEGA_BINARY, 0.0, 0.55), (O.OMEGA_LOGISTIC, 8.0, 0.5),
                                          (O.OMEGA_CLIP, 0.0, 0.0), (O.OMEGA_CONSTANT, 0.6, 0.0)])
def test_one_step_law_is_the_mixture(kind, a, delta):
    """Proposition 1 by simulation: draw a one-token step from P_m, score it,
    apply the criterion, fall back to a draw from P_M; the empirical law of
    the committed token must be omega_r P_m + nu P_M."""
    r = np.random.default_rng(11)
    V = 12
    lg_m, lg_M = r.normal(size=V), r.normal(size=V) + np.linspace(0, 1, V)
    rew = r.random(V)
    p_m, p_M = O.softmax(lg_m), O.softmax(lg_M)
    wts = np.array([O.omega(x, kind, delta, a) for x in rew])
    expect, nu = O.mixture_distribution(p_m, p_M, wts)
    n = 120000
    u = r.random((n, 3))
    counts = np.zeros(V)
    n_target = 0
    for i in range(n):
        y = O.sample(lg_m, u[i, 0], 1.0, 1.0)
        if not O.accept(rew[y], kind, delta, a, u[i, 1]):
            y = O.sample(lg_M, u[i, 2], 1.0, 1.0)
            n_target += 1
        counts[y] += 1
    chi2 = np.sum((counts - n * expect) ** 2 / (n * expect))
    assert chi2 < 40.0                                   # 11 dof: P(chi2 > 40) < 4e-5
    assert abs(n_target / n - nu) < 5 * np.sqrt(nu * (1 - nu) / n) + 1e-9


def test_expected_reward_does_not_drop_below_the_drafts():
    """Proposition 2 on random finite step sets: omega non-decreasing in r and
    E_{P_M}[r] >= E_{P_m}[r] imply E_{P_RSD}[r] >= E_{P_m}[r]."""
    r = np.random.default_rng(5)
    checked = 0
    for _ in range(300):
        V = 9
        rew = r.random(V)
        p_m, p_M = r.dirichlet(np.ones(V)), r.dirichlet(np.ones(V))
        if p_M @ rew < p_m @ rew:
            p_m, p_M = p_M, p_m
        kind = int(r.integers(0, 5))
        a = {O.OMEGA_CONSTANT: 0.4, O.OMEGA_LOGISTIC: 5.0}.get(kind, 0.0)
        wts = np.array([O.omega(x, kind, 0.5, a) for x in rew])
        mix, _ = O.mixture_distribution(p_m, p_M, wts)
        assert mix @ rew >= p_m @ rew - 1e-12
        checked += 1
    assert checked == 300


def test_full_loop_with_one_token_steps_follows_the_mixture(tiny):
    """The same law through the whole loop: step_cap = 1 makes every step one
    token, so the committed first token of a sequence is distributed as
    omega_r P_m + nu P_M with P_m, P_M and r read off the three models.  The
    vocabulary is cut to 8 ids (head rows of draft and target; the reward
    model's embedding rows are permuted to match) to keep the trial count low."""
    d, t, p = tiny["models"]
    ids = np.arange(8) * 100 + 3
    prompt = [int(x) for x in tiny["tokens"][0, :6]]
    assert min(prompt) >= len(ids)

    def restricted(m):
        wv = dict(m._w)
        wv["lm_head"] = m._w["lm_head"][ids]
        return O.OracleModel(m.s, wv)

    dm, tm = restricted(d), restricted(t)
    wp = dict(p._w)
    emb = np.array(p._w["embed"], copy=True)
    emb[:len(ids)] = p._w["embed"][ids]
    wp["embed"] = emb
    pm = O.OracleModel(p.s, wp)

    p_m = O.softmax(O.lm_logits(dm, O.forward_full(dm, prompt)[-1]))
    p_M = O.softmax(O.lm_logits(tm, O.forward_full(tm, prompt)[-1]))
    rew = np.array([O.reward(p, O.forward_full(p, prompt + [int(i)])[-1]) for i in ids])
    delta = float(np.float32(np.median(rew)))
    wts = np.array([O.omega(x, O.OMEGA_BINARY, delta) for x in rew])
    assert 0 < wts.sum() < len(ids)
    expect, nu = O.mixture_distribution(p_m, p_M, wts)

    P = O.Params(delta=delta, sep_id=0, step_cap=1, max_steps=1, max_ctx=len(prompt) + 1,
                 temperature=1.0, top_p=1.0)
    n = 3000
    r = np.random.default_rng(2)
    counts = np.zeros(len(ids))
    n_rej = 0
    for _ in range(n):
        out = O.generate_sequence(dm, tm, pm, prompt, r.random(len(prompt) + 1), r.random(len(prompt) + 1),
                                  np.zeros(1), P)
        counts[out["tokens"][-1]] += 1
        n_rej += not out["records"][0]["accepted"]
    chi2 = np.sum((counts - n * expect) ** 2 / (n * expect))
    assert chi2 < 35.0                                   # 7 dof: P(chi2 > 35) ~ 1e-5
    assert abs(n_rej / n - nu) < 5 * np.sqrt(nu * (1 - nu) / n)


# ------------------------------------------------------------ merged trunk (Appendix "Model Merge")
def merged_reward_model(policy, prm):
    """A reward model that shares every layer below the heads with `policy` and keeps `prm`'s own
    projection (cut or padded to the policy's width)."""
    from dataclasses import replace
    wv = {k: v for k, v in policy._w.items() if k != "lm_head"}
    d = policy.s.d_model
    w_r = np.zeros(d, np.float32)
    n = min(d, prm._w["w_r"].size)
    w_r[:n] = prm._w["w_r"][:n] * 40.0            # spread the rewards around 1/2 (the head is N(0, 0.02))
    wv["w_r"], wv["b_r"] = w_r, prm._w["b_r"]
    return O.OracleModel(replace(policy.s, head_kind=prm.s.head_kind), wv)


@pytest.mark.parametrize("which", ["draft", "target"])
def test_merged_trunk_equals_a_separate_reward_model_with_the_same_layers(tiny, which):
    """With the reward head on a policy model's trunk the loop must produce what it produces with a
    separate third model whose layers are copies of that trunk: the merged run reads the reward off
    the policy model's own incremental forward, the separate run off an independent model with its
    own cache fed in different chunks."""
    d, t, p = tiny["models"]
    pm = merged_reward_model(d if which == "draft" else t, p)
    P = params(tiny["w"], temperature=0.7, top_p=0.95, sep_logit_bias=3.5, delta=0.5)
    from dataclasses import replace
    first = [run(tiny, b, P, models=(d, t, pm), max_steps=1)["records"][0]["reward"] for b in range(4)]
    P = replace(P, delta=float(np.median(first)))             # a threshold that both accepts and rejects
    n_acc = n_rej = 0
    for b in range(4):
        a = run(tiny, b, P, models=(d, t, pm))
        m = run(tiny, b, replace(P, merge=which), models=(d, t, pm))
        assert a["tokens"] == m["tokens"]
        for ra, rm in zip(a["records"], m["records"]):
            assert abs(ra["reward"] - rm["reward"]) < 1e-12
            assert ra["accepted"] == rm["accepted"] and ra["final_tokens"] == rm["final_tokens"]
            ctx = rm["ctx_len"]
            assert rm["kv_len"][2] == 0                              # no third cache
            assert rm["kv_len"][0] == (ctx - 1 if rm["accepted"] else rm["ctx_pre"])
            if which == "target":
                assert rm["kv_len"][1] == ctx - 1                    # the target has read every step
            else:
                assert rm["kv_len"][1] == ra["kv_len"][1]
            n_acc += rm["accepted"]; n_rej += not rm["accepted"]
    assert n_acc >= 2 and n_rej >= 2
